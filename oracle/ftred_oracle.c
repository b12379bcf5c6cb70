/*
 * CPU oracle for the correction-based fault-tolerant reduce and allreduce
 * (Kuettler & Haertig, "Fault-tolerant Reduce and Allreduce operations based on
 * correction").
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, literal
 * simulation: one object per process, one message queue per process, explicit
 * adjacency lists, a global round loop.  It exists so that the GPU library can
 * be checked against something that can be compared with the paper by eye.
 * It shares no code, header, table or constant with the GPU library.
 *
 * What follows the paper directly:
 *   - root relabelling by swapping the root's number with 0      (section "Reduce")
 *   - up-correction groups by group number floor((p-1)/(f+1)); the root joins
 *     the last group iff that group is short          (section "Up-Correction")
 *   - Algorithm "Up-correction": every member sends its ORIGINAL input to every
 *     other member and folds what it receives; no failure information is sent
 *   - Algorithm "reduce, non-roots": up-correction, then receive from all
 *     children, fold, update failure information, send to parent
 *   - Algorithm "reduce, root": optional up-correction, then take a child
 *     message that reports no failure; add the root's value iff the sender's
 *     subtree does not already contain it
 *   - failure information: the single "failed" bit, set in the tree phase when
 *     a child's value is missing, untouched in up-correction
 *                                             (section "Failure information")
 *   - the two richer schemes of the same section (entry points *_info): every
 *     process appends the id of each process it cannot receive a value from,
 *     in the up-correction phase and in the tree phase, to a list; the list
 *     travels with the tree message and a parent adds its children's lists to
 *     its own (first scheme); only the length of that list travels (second
 *     scheme).  Both are tracked side by side; which child the root selects
 *     depends on the failed bit alone, so the value is the same in all schemes.
 *     Reported: list and length carried by the message the root selects.
 *   - I(f)-tree: the root has f+1 children whose subtrees differ in size by at
 *     most one; process a is in subtree k iff (a-1) mod (f+1) == k-1
 *                                  (Definition and proof of the first theorem)
 *   - Algorithm "Allreduce": r <- 0; repeat { reduce to r; broadcast from r;
 *     ok <- broadcast succeeded; r <- successor(r) }
 *
 * Readings taken where the paper is silent (each is also listed in the design
 * notes of the repository):
 *   R1 round model: global rounds 1,2,...; a message sent in round r reaches an
 *      alive receiver at the end of round r.  Every message has the round it has
 *      in the failure-free run; a message that is absent at the end of that
 *      round means "sender failed" (stands for time-out + failure monitor).
 *      fail_round 0 = failed before the operation; fail_round r >= 1 = the
 *      process does everything of rounds < r and nothing from round r on.
 *   R2 up-correction order: in round t (1..f) the member with index i of a group
 *      of size g sends to index (i+t) mod g iff t <= g-1.
 *   R3 tree inside a root subtree: filled breadth-first, two children per node
 *      (the default).  The definition of the I(f)-tree fixes only the root's
 *      f+1 children and the sizes of their subtrees, so other shapes are offered
 *      (entry points *_shape*): k children per node, filled breadth-first, and
 *      the binomial tree built by doubling.
 *   R4 a tree process sends in round f + 1 + height(process).
 *   R5 root choice among child messages: lowest child number whose message is
 *      present and reports no failure.
 *   R6 allreduce roots: physical ranks 0,1,...,f in this order; they may fail
 *      only before the operation.
 *   R7 broadcast (defined in a companion paper, not available): tree-down over
 *      the same tree (D rounds), then f correction rounds in which every holder
 *      sends the value to group mate (i+t) mod g.
 *
 *   R8 latency bookkeeping (the paper gives no cost model; section "Up-Correction"
 *      says a receiver times out on a failed sender and asks the failure
 *      monitor): a process is DETECTED when a process that is alive finds, in
 *      the round in which it acts on it, that a message of the failure-free
 *      schedule has not come, and the monitor (the failure list) says the sender
 *      has failed.  A round COSTS as many message steps as the busiest process
 *      sends or receives messages in it in the failure-free run (one port per
 *      process).  Both are counted literally by the simulation.
 *   R9 event-driven times of the reduce (section "Related work", last
 *      paragraph: a process runs its phases one after the other without regard
 *      to the progress of the others; section "Up-Correction", last paragraph,
 *      and the liveness part of the proof in "Reduce / Properties": a receive
 *      from a failed sender ends by a time-out and the monitor's confirmation,
 *      and is retried while the monitor says the sender lives).  Every process
 *      starts at time 0 and has a clock of its own.  A send takes t_msg of the
 *      sender's time and the message is at the receiver when the send ends.  A
 *      receive ends at once if the message is there, at its arrival otherwise;
 *      if the sender has stopped without sending it, the receiver asks the
 *      monitor after every t_timeout of waiting and gives up at the first such
 *      moment that lies after the moment the sender stopped.  A process stops
 *      when it reaches the first step whose round (R1, R4) is >= its
 *      fail_round; what is sent and received, hence every value, status and
 *      message count, is that of the round model, because a process awaits
 *      named senders in a fixed order (R2, R5) and never whoever comes first.
 *      The simulation stamps these times onto its round loop (entry point
 *      oracle_reduce_timed_batch); event_sim.py beside this file runs the same
 *      model as a discrete-event simulation with blocking receives and pins it.
 *
 * parity pins: every function of this file is pinned by tests (worked example
 * of the paper, brute force over all failure subsets against the survivor
 * reduction, one-hot multiplicities, message-count closed forms).  Not pinned by
 * the paper (they are this repository's definitions): the number of rounds, the
 * choice among valid results under in-operation failures, and the broadcast's
 * message counts.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_NO_RANK 0xFFFFFFFFu
#define ORACLE_NEVER UINT64_MAX

enum { OR_I64 = 0, OR_U32 = 1, OR_F64 = 2 };
enum { OR_SUM = 0, OR_BOR = 1 };
enum {
    OR_ST_OK = 0,
    OR_ST_ROOT_FAILED = 1,
    OR_ST_NO_CLEAN_SUBTREE = 2,
    OR_ST_BAD_FAILURE_SET = 3,
    OR_ST_INCONSISTENT = 4,
    OR_ST_NO_LIVE_ROOT = 5
};
enum { MSG_UC = 0, MSG_TREE = 1, MSG_BCAST = 2, MSG_BCORR = 3 };

/* ------------------------------------------------------------------ */
/* reduction function                                                   */

static size_t elem_size(int dtype)
{
    return dtype == OR_U32 ? 4 : 8;
}

/* dst <- reduce_function(dst, src), element by element */
static void combine(int dtype, int op, uint32_t elems, void *dst, const void *src)
{
    uint32_t e;
    if (dtype == OR_F64) {
        double *d = (double *)dst;
        const double *s = (const double *)src;
        for (e = 0; e < elems; ++e) d[e] = d[e] + s[e];
    } else if (dtype == OR_I64) {
        /* wrapping sum: done on the unsigned representation */
        uint64_t *d = (uint64_t *)dst;
        const uint64_t *s = (const uint64_t *)src;
        for (e = 0; e < elems; ++e) d[e] = (op == OR_SUM) ? d[e] + s[e] : (d[e] | s[e]);
    } else {
        uint32_t *d = (uint32_t *)dst;
        const uint32_t *s = (const uint32_t *)src;
        for (e = 0; e < elems; ++e) d[e] = (op == OR_SUM) ? d[e] + s[e] : (d[e] | s[e]);
    }
}

/* ------------------------------------------------------------------ */
/* structure: built constructively, with explicit lists                 */

typedef struct {
    uint32_t P, f, root;
    uint32_t *phys_of_virt;   /* [P] */
    uint32_t *virt_of_phys;   /* [P] */
    int64_t *parent;          /* [P] virtual parent, -1 for the root */
    uint32_t *nkids;          /* [P] */
    uint32_t *kid_off;        /* [P+1] children of non-root v: kids[kid_off[v] .. kid_off[v] + nkids[v]) in the order they joined */
    uint32_t *kids;           /* [P] */
    uint32_t *root_kids;      /* [f+1] */
    int shape;                /* see topo_build */
    uint32_t *subtree;        /* [P] 0 for the root, else 1..f+1 */
    int64_t *group;           /* [P] group id or -1 */
    uint32_t *gpos;           /* [P] index in the group's member list */
    uint32_t ngroups;
    uint32_t *gsize;          /* [ngroups] */
    uint32_t *gmembers;       /* [ngroups][f+2] */
    uint32_t *height;         /* [P] */
    uint32_t *depth;          /* [P] */
    uint32_t D;               /* height of the root */
} topo_t;

static void topo_free(topo_t *t)
{
    free(t->phys_of_virt); free(t->virt_of_phys); free(t->parent); free(t->nkids);
    free(t->kids); free(t->kid_off); free(t->root_kids); free(t->subtree); free(t->group); free(t->gpos);
    free(t->gsize); free(t->gmembers); free(t->height); free(t->depth);
    memset(t, 0, sizeof(*t));
}

/* shape of the tree inside each subtree of the root (the definition of the I(f)-tree leaves it free):
     k >= 2  k children per process, filled breadth-first: the next process of a subtree becomes a child of the
             oldest process of that subtree with fewer than k children (k = 2 is the tree of the paper's second
             tree figure and the default everywhere)
     1       binomial tree built by doubling: the process that joins a subtree as its j-th (j >= 1, the first
             one is number 0) becomes a child of the one that joined as number j - 2^floor(log2 j) */
#define SHAPE_BINOMIAL 1
#define SHAPE_DEFAULT 2

static int topo_build(topo_t *t, uint32_t P, uint32_t f, uint32_t root, int shape)
{
    uint32_t v, k, nsub = f + 1, gcap = f + 2, cap;
    uint32_t *open_head, *open_tail, *open_next, *sub_count, *joined, *fill;
    memset(t, 0, sizeof(*t));
    if (P < f + 2 || root >= P || shape < 1 || shape > 64) return -1;
    t->P = P; t->f = f; t->root = root; t->shape = shape;
    t->phys_of_virt = malloc(sizeof(uint32_t) * P);
    t->virt_of_phys = malloc(sizeof(uint32_t) * P);
    t->parent = malloc(sizeof(int64_t) * P);
    t->nkids = calloc(P, sizeof(uint32_t));
    t->kid_off = calloc((size_t)P + 1, sizeof(uint32_t));
    t->kids = calloc((size_t)P, sizeof(uint32_t));
    t->root_kids = calloc(nsub, sizeof(uint32_t));
    t->subtree = calloc(P, sizeof(uint32_t));
    t->group = malloc(sizeof(int64_t) * P);
    t->gpos = calloc(P, sizeof(uint32_t));
    t->ngroups = (P - 1) / (f + 1) + 1;
    t->gsize = calloc(t->ngroups, sizeof(uint32_t));
    t->gmembers = calloc((size_t)t->ngroups * gcap, sizeof(uint32_t));
    t->height = calloc(P, sizeof(uint32_t));
    t->depth = calloc(P, sizeof(uint32_t));

    /* the root's number is swapped with 0 */
    for (v = 0; v < P; ++v) t->phys_of_virt[v] = v;
    t->phys_of_virt[0] = root;
    t->phys_of_virt[root] = 0;
    if (root == 0) t->phys_of_virt[0] = 0;
    for (v = 0; v < P; ++v) t->virt_of_phys[t->phys_of_virt[v]] = v;

    /* I(f)-tree: deal 1..P-1 round-robin to f+1 subtrees; the first process of a subtree is a child of the
       root, every later one gets its parent inside the subtree by the rule of the shape */
    cap = (P - 1 + nsub - 1) / nsub;               /* most processes in one subtree */
    open_head = malloc(sizeof(uint32_t) * nsub);   /* oldest process with a free slot (breadth-first shapes) */
    open_tail = malloc(sizeof(uint32_t) * nsub);
    open_next = calloc(P, sizeof(uint32_t));       /* queue links */
    sub_count = calloc(nsub, sizeof(uint32_t));
    joined = calloc((size_t)nsub * cap, sizeof(uint32_t));   /* [subtree][number of joining] -> process */
    t->parent[0] = -1;
    t->nkids[0] = 0;
    k = 0;
    for (v = 1; v < P; ++v) {
        const uint32_t jn = sub_count[k];          /* v joins its subtree as number jn */
        t->subtree[v] = k + 1;
        joined[(size_t)k * cap + jn] = v;
        if (jn == 0) {
            t->parent[v] = 0;
            t->root_kids[t->nkids[0]++] = v;
            open_head[k] = v;
        } else if (shape == SHAPE_BINOMIAL) {
            uint32_t top = 1;
            while (2 * top <= jn) top *= 2;        /* 2^floor(log2 jn) */
            t->parent[v] = joined[(size_t)k * cap + (jn - top)];
            t->nkids[t->parent[v]]++;
        } else {
            uint32_t p = open_head[k];
            t->parent[v] = p;
            t->nkids[p]++;
            if (t->nkids[p] == (uint32_t)shape) open_head[k] = open_next[p];
            open_next[open_tail[k]] = v;
        }
        open_tail[k] = v;
        sub_count[k]++;
        k = (k + 1) % nsub;
    }
    free(open_head); free(open_tail); free(open_next); free(sub_count); free(joined);
    /* the lists of children, each in the order in which the children joined (ascending numbers) */
    for (v = 1; v < P; ++v) t->kid_off[v + 1] = t->kid_off[v] + t->nkids[v];
    fill = calloc(P, sizeof(uint32_t));
    for (v = 1; v < P; ++v)
        if (t->parent[v] > 0) {
            uint32_t p = (uint32_t)t->parent[v];
            t->kids[t->kid_off[p] + fill[p]++] = v;
        }
    free(fill);

    /* up-correction groups: consecutive runs of f+1 processes; a short last
       run takes the root as its last member */
    for (v = 0; v < P; ++v) t->group[v] = -1;
    {
        uint32_t g = 0;
        for (v = 1; v < P; ++v) {
            t->group[v] = g;
            t->gpos[v] = t->gsize[g];
            t->gmembers[(size_t)g * gcap + t->gsize[g]++] = v;
            if (t->gsize[g] == f + 1) ++g;
        }
        if (g < t->ngroups && t->gsize[g] > 0 && t->gsize[g] < f + 1) {
            t->group[0] = g;
            t->gpos[0] = t->gsize[g];
            t->gmembers[(size_t)g * gcap + t->gsize[g]++] = 0;
            ++g;
        }
        t->ngroups = g;
    }

    /* depth and height from the explicit parent links (children have larger
       numbers than their parents) */
    for (v = 1; v < P; ++v) t->depth[v] = t->depth[t->parent[v]] + 1;
    for (v = P - 1; v >= 1; --v) {
        uint32_t p = (uint32_t)t->parent[v];
        if (t->height[p] < t->height[v] + 1) t->height[p] = t->height[v] + 1;
    }
    t->D = t->height[0];
    return 0;
}

/* ------------------------------------------------------------------ */
/* processes, messages, network                                         */

typedef struct msg {
    struct msg *next;
    int kind;
    uint32_t src, dst;       /* virtual ranks */
    int flag;                /* failure information: the single failed bit */
    uint32_t count;          /* second scheme: length of the sender's list */
    uint32_t nids;           /* first scheme: the list itself (virtual ranks) */
    uint32_t *ids;
    unsigned char *data;
    uint64_t time;           /* timed mode (R9): the moment the message is at the receiver */
} msg_t;

typedef struct {
    msg_t *head, *tail;      /* inbox: FIFO queue */
} inbox_t;

typedef struct {
    const topo_t *t;
    uint32_t elems; int dtype, op;
    size_t bytes;            /* bytes of one value */
    uint32_t nfail;
    const uint32_t *fail_virt;   /* [nfail] virtual ranks (ORACLE_NO_RANK = unused) */
    const uint32_t *fail_round;  /* [nfail] */
    unsigned char *input;    /* [P][bytes] by virtual rank */
    unsigned char *data;     /* [P][bytes] working value of each process */
    inbox_t *inbox;          /* [P] */
    msg_t *inflight_head, *inflight_tail;
    /* arena for messages */
    unsigned char *arena; size_t arena_used, arena_cap;
    uint64_t sent[4];
    /* latency bookkeeping (R8) */
    uint32_t detected;       /* bit q: the process in slot q of the failure list was detected as failed */
    int count_steps;         /* count the message steps of every round */
    uint32_t steps[4];       /* per kind of message: sum over the rounds of the busiest process's messages */
    uint32_t *port_in, *port_out;   /* [P] scratch of count_steps */
    /* event-driven times of the reduce (R9); tracked iff timed */
    int timed;
    uint64_t t_msg, t_timeout;
    uint64_t *clock;         /* [P] each process's own time: advances by its sends and its waits only */
    uint64_t *finish;        /* [P] the moment a process has done its part; ORACLE_NEVER while it has not */
    uint64_t t_done;         /* the moment the root delivers (or gives up) */
    /* broadcast state */
    unsigned char *has;      /* [P] */
    unsigned char *held;     /* [P][bytes] */
    /* traces (by virtual rank) */
    unsigned char *trace_v;  /* [P][bytes] or NULL */
    unsigned char *trace_sent, *trace_flag; /* [P] or NULL */
    unsigned char *trace_msg; /* [P][bytes] or NULL */
    int disable_uc;
    /* failure information, first and second scheme (tracked iff track_info) */
    int track_info;
    uint32_t flcap;          /* capacity of one list */
    uint32_t *fl;            /* [P][flcap] ids a process could not receive a value from, and its children's lists */
    uint32_t *fn;            /* [P] entries in fl */
    uint32_t *fcount;        /* [P] the counter of the second scheme */
    int info_overflow;       /* a list outgrew flcap (never, if concatenated lists are disjoint) */
    uint32_t sel_count, sel_nids, sel_child;
    uint32_t *sel_ids;       /* [flcap] list carried by the message the root selected */
    /* what the root holds from each of its f+1 children at the end: state 0 = no message,
       1 = message without the failed bit, 2 = message with the failed bit */
    uint32_t *ch_state, *ch_count, *ch_nids, *ch_ids;   /* [f+1], [f+1], [f+1], [f+1][flcap] */
} sim_t;

static int alive(const sim_t *s, uint32_t v, uint32_t round)
{
    uint32_t i;
    for (i = 0; i < s->nfail; ++i)
        if (s->fail_virt[i] == v)
            return s->fail_round[i] != 0 && round < s->fail_round[i];
    return 1;
}

static void *arena_alloc(sim_t *s, size_t n)
{
    void *p;
    n = (n + 15) & ~(size_t)15;
    if (s->arena_used + n > s->arena_cap) {
        /* chain a new block; old blocks are leaked into a list */
        size_t cap = s->arena_cap ? s->arena_cap : ((size_t)1 << 20);
        unsigned char *blk;
        while (cap < n + 16) cap *= 2;
        blk = malloc(cap + 16);
        *(unsigned char **)blk = s->arena;   /* link to previous block base */
        s->arena = blk;
        s->arena_used = 16;
        s->arena_cap = cap + 16;
    }
    p = s->arena + s->arena_used;
    s->arena_used += n;
    return p;
}

static void arena_release(sim_t *s)
{
    while (s->arena) {
        unsigned char *prev = *(unsigned char **)s->arena;
        free(s->arena);
        s->arena = prev;
    }
    s->arena_used = s->arena_cap = 0;
}

/* send: completes whether or not the destination is alive */
static void net_send(sim_t *s, int kind, uint32_t src, uint32_t dst, const void *data, int flag)
{
    msg_t *m = arena_alloc(s, sizeof(msg_t));
    m->next = NULL; m->kind = kind; m->src = src; m->dst = dst; m->flag = flag;
    m->count = 0; m->nids = 0; m->ids = NULL;
    if (s->track_info && kind == MSG_TREE) {
        /* the sender's list (first scheme) and its length counter (second scheme) */
        m->count = s->fcount[src];
        m->nids = s->fn[src];
        m->ids = arena_alloc(s, sizeof(uint32_t) * (m->nids + 1));
        memcpy(m->ids, s->fl + (size_t)src * s->flcap, sizeof(uint32_t) * m->nids);
    }
    m->data = arena_alloc(s, s->bytes);
    memcpy(m->data, data, s->bytes);
    m->time = 0;
    if (s->timed) {
        /* the send takes t_msg of the sender's time; the message is at the receiver when the send ends */
        s->clock[src] += s->t_msg;
        m->time = s->clock[src];
    }
    if (s->inflight_tail) s->inflight_tail->next = m; else s->inflight_head = m;
    s->inflight_tail = m;
    s->sent[kind]++;
}

/* Timed mode (R9).  Process v takes the message m it was waiting for: at once if it is there already, at its
   arrival otherwise. */
static void clock_receive(sim_t *s, uint32_t v, const msg_t *m)
{
    if (s->timed && m->time > s->clock[v]) s->clock[v] = m->time;
}

/* Timed mode (R9).  Process v waits for a message of process u that never comes (u has stopped: its clock stands
   at that moment).  After every t_timeout of waiting v asks the monitor and gives up at the first such moment
   that lies after the moment u stopped. */
static void clock_give_up(sim_t *s, uint32_t v, uint32_t u)
{
    uint64_t k = 1;
    if (!s->timed) return;
    if (s->clock[u] >= s->clock[v] + s->t_timeout) k = (s->clock[u] - s->clock[v]) / s->t_timeout + 1;
    s->clock[v] += k * s->t_timeout;
}

/* A process that is alive has waited in vain for a message of process u that was due by now: it asks the
   failure monitor, and if u has failed, u counts as detected (R8). */
static void monitor_query(sim_t *s, uint32_t u, uint32_t now)
{
    uint32_t i;
    if (alive(s, u, now)) return;
    for (i = 0; i < s->nfail && i < 32; ++i)
        if (s->fail_virt[i] == u) s->detected |= 1u << i;
}

/* end of a round: messages reach the inboxes of processes alive in this round;
   a failed process gives no reaction to a message */
static void net_deliver(sim_t *s, uint32_t round)
{
    msg_t *m = s->inflight_head;
    if (s->count_steps && m) {
        /* one port per process: the round takes as many message steps as the busiest process sends or receives */
        uint32_t most = 0;
        int kind = m->kind;
        msg_t *q;
        for (q = m; q; q = q->next) {
            if (++s->port_out[q->src] > most) most = s->port_out[q->src];
            if (++s->port_in[q->dst] > most) most = s->port_in[q->dst];
        }
        for (q = m; q; q = q->next) s->port_out[q->src] = s->port_in[q->dst] = 0;
        s->steps[kind] += most;
    }
    while (m) {
        msg_t *nx = m->next;
        m->next = NULL;
        if (alive(s, m->dst, round)) {
            inbox_t *q = &s->inbox[m->dst];
            if (q->tail) q->tail->next = m; else q->head = m;
            q->tail = m;
        }
        m = nx;
    }
    s->inflight_head = s->inflight_tail = NULL;
}

/* remove and return the first message of this kind from src (or NULL) */
static msg_t *inbox_take(sim_t *s, uint32_t v, int kind, uint32_t src)
{
    inbox_t *q = &s->inbox[v];
    msg_t *prev = NULL, *m = q->head;
    while (m) {
        if (m->kind == kind && m->src == src) {
            if (prev) prev->next = m->next; else q->head = m->next;
            if (q->tail == m) q->tail = prev;
            m->next = NULL;
            return m;
        }
        prev = m; m = m->next;
    }
    return NULL;
}

/* the first message of this kind from src, left in the inbox (or NULL) */
static const msg_t *inbox_peek(const sim_t *s, uint32_t v, int kind, uint32_t src)
{
    const msg_t *m = s->inbox[v].head;
    while (m && !(m->kind == kind && m->src == src)) m = m->next;
    return m;
}

/* remove and return the first message of this kind (any sender) */
static msg_t *inbox_take_any(sim_t *s, uint32_t v, int kind)
{
    inbox_t *q = &s->inbox[v];
    msg_t *prev = NULL, *m = q->head;
    while (m) {
        if (m->kind == kind) {
            if (prev) prev->next = m->next; else q->head = m->next;
            if (q->tail == m) q->tail = prev;
            m->next = NULL;
            return m;
        }
        prev = m; m = m->next;
    }
    return NULL;
}

/* process v could not receive a value from process id: append it to v's list */
static void info_append(sim_t *s, uint32_t v, uint32_t id)
{
    if (s->fn[v] < s->flcap) s->fl[(size_t)v * s->flcap + s->fn[v]++] = id;
    else s->info_overflow = 1;
}

static void clear_inboxes(sim_t *s)
{
    uint32_t v;
    for (v = 0; v < s->t->P; ++v) s->inbox[v].head = s->inbox[v].tail = NULL;
    s->inflight_head = s->inflight_tail = NULL;
}

/* ------------------------------------------------------------------ */
/* who exchanges with whom inside a group (R2, R7)                      */

/* up-correction round r (1 <= r <= group size - 1): the mate v sends its input to, and the mate v hears from */
static uint32_t uc_target(const topo_t *t, uint32_t v, uint32_t r)
{
    const uint32_t g = (uint32_t)t->group[v], gs = t->gsize[g];
    return t->gmembers[(size_t)g * (t->f + 2) + (t->gpos[v] + r) % gs];
}

static uint32_t uc_source(const topo_t *t, uint32_t v, uint32_t r)
{
    const uint32_t g = (uint32_t)t->group[v], gs = t->gsize[g];
    return t->gmembers[(size_t)g * (t->f + 2) + (t->gpos[v] + gs - r) % gs];
}

/* correction round tt of the broadcast: the same rotation here (R7); the one place to change for another
   correction scheme, e.g. the corrected-tree broadcast of the companion paper */
static uint32_t correction_target(const topo_t *t, uint32_t v, uint32_t tt) { return uc_target(t, v, tt); }
static uint32_t correction_source(const topo_t *t, uint32_t v, uint32_t tt) { return uc_source(t, v, tt); }

/* ------------------------------------------------------------------ */
/* one reduce to virtual rank 0, global rounds base+1 .. base+f+D        */
/* returns the per-operation status; result (bytes) valid when OK        */

static int run_reduce(sim_t *s, uint32_t base, void *result)
{
    const topo_t *t = s->t;
    const uint32_t P = t->P, f = t->f, gcap = t->f + 2;
    const uint32_t R = f + t->D;
    uint32_t r, v, c;
    unsigned char *fold = malloc(s->bytes);

    /* every process starts from its input; "senddata" is the input itself */
    memcpy(s->data, s->input, (size_t)P * s->bytes);
    clear_inboxes(s);
    if (s->track_info) {
        memset(s->fn, 0, sizeof(uint32_t) * P);
        memset(s->fcount, 0, sizeof(uint32_t) * P);
        s->sel_count = s->sel_nids = 0;
    }

    for (r = 1; r <= R; ++r) {
        const uint32_t now = base + r;
        /* --- sends of this round, from the state at the start of the round --- */
        for (v = 0; v < P; ++v) {
            if (!alive(s, v, now)) continue;
            if (r <= f) {
                /* up-correction round t = r */
                if (!s->disable_uc && t->group[v] >= 0) {
                    uint32_t g = (uint32_t)t->group[v], gs = t->gsize[g];
                    if (r <= gs - 1)
                        net_send(s, MSG_UC, v, uc_target(t, v, r), s->input + (size_t)v * s->bytes, 0);
                }
            } else if (v != 0 && r == f + 1 + t->height[v]) {
                /* tree phase: all children had their turn; fold and send up */
                int flag = 0;
                memcpy(fold, s->data + (size_t)v * s->bytes, s->bytes);
                for (c = 0; c < t->nkids[v]; ++c) {
                    msg_t *m = inbox_take(s, v, MSG_TREE, t->kids[t->kid_off[v] + c]);
                    if (m) {
                        combine(s->dtype, s->op, s->elems, fold, m->data);
                        clock_receive(s, v, m);
                        if (m->flag) flag = 1;
                        if (s->track_info) {       /* the parent adds the child's list to its own */
                            uint32_t i;
                            for (i = 0; i < m->nids; ++i) info_append(s, v, m->ids[i]);
                            s->fcount[v] += m->count;
                        }
                    } else {
                        flag = 1;    /* no value from this child */
                        monitor_query(s, t->kids[t->kid_off[v] + c], now);
                        clock_give_up(s, v, t->kids[t->kid_off[v] + c]);
                        if (s->track_info) {
                            info_append(s, v, t->kids[t->kid_off[v] + c]);
                            s->fcount[v] += 1;
                        }
                    }
                }
                net_send(s, MSG_TREE, v, (uint32_t)t->parent[v], fold, flag);
                if (s->timed) s->finish[v] = s->clock[v];
                if (s->trace_sent) s->trace_sent[v] = 1;
                if (s->trace_flag) s->trace_flag[v] = (unsigned char)flag;
                if (s->trace_msg) memcpy(s->trace_msg + (size_t)v * s->bytes, fold, s->bytes);
            }
        }
        /* --- end of round: deliveries, then receivers act --- */
        net_deliver(s, now);
        if (r <= f) {
            for (v = 0; v < P; ++v) {
                msg_t *m;
                int got = 0;
                if (!alive(s, v, now)) continue;
                while ((m = inbox_take_any(s, v, MSG_UC)) != NULL) {
                    combine(s->dtype, s->op, s->elems, s->data + (size_t)v * s->bytes, m->data);
                    clock_receive(s, v, m);
                    got = 1;
                }
                if (!s->disable_uc && t->group[v] >= 0 && !got) {
                    /* the member that sends to v in this round (R2) sent nothing */
                    uint32_t g = (uint32_t)t->group[v], gs = t->gsize[g];
                    if (r <= gs - 1) {
                        uint32_t mate = uc_source(t, v, r);
                        monitor_query(s, mate, now);
                        clock_give_up(s, v, mate);
                        if (s->track_info) {
                            info_append(s, v, mate);
                            s->fcount[v] += 1;
                        }
                    }
                }
            }
        }
        if (r == f && s->trace_v) memcpy(s->trace_v, s->data, (size_t)P * s->bytes);
    }
    if (f == 0 && s->trace_v) memcpy(s->trace_v, s->data, (size_t)P * s->bytes);
    free(fold);

    /* --- the root, at the end of the last round --- */
    if (!alive(s, 0, base + R)) return OR_ST_ROOT_FAILED;
    for (c = 0; c < t->nkids[0]; ++c)      /* every child's message was due by now */
        if (!inbox_peek(s, 0, MSG_TREE, t->root_kids[c])) monitor_query(s, t->root_kids[c], base + R);
    if (s->track_info) {
        /* the failure information the root received, child by child */
        for (c = 0; c < t->nkids[0]; ++c) {
            const msg_t *m = inbox_peek(s, 0, MSG_TREE, t->root_kids[c]);
            s->ch_state[c] = !m ? 0u : (m->flag ? 2u : 1u);
            s->ch_count[c] = m ? m->count : 0u;
            s->ch_nids[c] = m ? m->nids : 0u;
            if (m) memcpy(s->ch_ids + (size_t)c * s->flcap, m->ids, sizeof(uint32_t) * m->nids);
        }
    }
    for (c = 0; c < t->nkids[0]; ++c) {
        uint32_t child = t->root_kids[c];
        msg_t *m = inbox_take(s, 0, MSG_TREE, child);
        int included = 0;
        uint32_t i;
        /* the root takes its children in order and stops at the first it can use */
        if (m) clock_receive(s, 0, m); else clock_give_up(s, 0, child);
        if (s->timed) s->t_done = s->finish[0] = s->clock[0];
        if (!m || m->flag) continue;      /* absent, or failure in that subtree */
        /* is the root's value already in this message?  Yes iff the sender's
           subtree holds a member of the root's up-correction group. */
        if (!s->disable_uc && t->group[0] >= 0) {
            uint32_t g = (uint32_t)t->group[0];
            for (i = 0; i < t->gsize[g]; ++i) {
                uint32_t mem = t->gmembers[(size_t)g * gcap + i];
                if (mem != 0 && t->subtree[mem] == t->subtree[child]) included = 1;
            }
        }
        if (included) {
            memcpy(result, m->data, s->bytes);
        } else {
            memcpy(result, s->data, s->bytes);                   /* the root's value */
            combine(s->dtype, s->op, s->elems, result, m->data);
        }
        if (s->track_info) {
            s->sel_child = c;
            s->sel_count = m->count;
            s->sel_nids = m->nids;
            memcpy(s->sel_ids, m->ids, sizeof(uint32_t) * m->nids);
        }
        return OR_ST_OK;
    }
    return OR_ST_NO_CLEAN_SUBTREE;
}

/* broadcast of `value` from virtual rank 0, rounds base+1 .. base+D+f */
static void run_broadcast(sim_t *s, uint32_t base, const void *value)
{
    const topo_t *t = s->t;
    const uint32_t P = t->P, f = t->f;
    uint32_t r, v, c;
    clear_inboxes(s);
    memset(s->has, 0, P);
    s->has[0] = 1;
    memcpy(s->held, value, s->bytes);
    for (r = 1; r <= t->D + f; ++r) {
        const uint32_t now = base + r;
        for (v = 0; v < P; ++v) {
            if (!alive(s, v, now) || !s->has[v]) continue;
            if (r <= t->D) {
                /* tree-down: depth r-1 sends to all its children */
                if (t->depth[v] != r - 1) continue;
                if (v == 0) {
                    for (c = 0; c < t->nkids[0]; ++c)
                        net_send(s, MSG_BCAST, 0, t->root_kids[c], s->held, 0);
                } else {
                    for (c = 0; c < t->nkids[v]; ++c)
                        net_send(s, MSG_BCAST, v, t->kids[t->kid_off[v] + c],
                                 s->held + (size_t)v * s->bytes, 0);
                }
            } else if (t->group[v] >= 0) {
                /* correction round tt: every holder sends to one group mate */
                uint32_t tt = r - t->D;
                uint32_t g = (uint32_t)t->group[v], gs = t->gsize[g];
                if (tt <= gs - 1)
                    net_send(s, MSG_BCORR, v, correction_target(t, v, tt), s->held + (size_t)v * s->bytes, 0);
            }
        }
        net_deliver(s, now);
        for (v = 0; v < P; ++v) {
            msg_t *m;
            if (!alive(s, v, now)) continue;
            /* the message of the failure-free schedule for v in this round: from its parent when the value
               reaches v's depth, from one group mate in a correction round */
            if (r <= t->D) {
                if (v != 0 && t->depth[v] == r && !inbox_peek(s, v, MSG_BCAST, (uint32_t)t->parent[v]))
                    monitor_query(s, (uint32_t)t->parent[v], now);
            } else if (t->group[v] >= 0) {
                uint32_t tt = r - t->D;
                uint32_t g = (uint32_t)t->group[v], gs = t->gsize[g];
                if (tt <= gs - 1) {
                    uint32_t mate = correction_source(t, v, tt);
                    if (!inbox_peek(s, v, MSG_BCORR, mate)) monitor_query(s, mate, now);
                }
            }
            while ((m = inbox_take_any(s, v, r <= t->D ? MSG_BCAST : MSG_BCORR)) != NULL) {
                if (!s->has[v]) {       /* keep the first value */
                    s->has[v] = 1;
                    memcpy(s->held + (size_t)v * s->bytes, m->data, s->bytes);
                }
            }
        }
    }
}

/* ------------------------------------------------------------------ */
/* set-up shared by the entry points                                    */

static int check_failures(uint32_t P, uint32_t nfail, const uint32_t *fail_rank)
{
    uint32_t i, j;
    for (i = 0; i < nfail; ++i) {
        if (fail_rank[i] == ORACLE_NO_RANK) continue;
        if (fail_rank[i] >= P) return -1;
        for (j = 0; j < i; ++j)
            if (fail_rank[j] == fail_rank[i]) return -1;
    }
    return 0;
}

static void sim_init(sim_t *s, const topo_t *t, uint32_t elems, int dtype, int op,
                     const void *payload /* by physical rank */,
                     uint32_t nfail, const uint32_t *fail_rank, const uint32_t *fail_round,
                     uint32_t *fail_virt_buf)
{
    uint32_t v, i;
    memset(s, 0, sizeof(*s));
    s->t = t; s->elems = elems; s->dtype = dtype; s->op = op;
    s->bytes = elems * elem_size(dtype);
    s->nfail = nfail;
    for (i = 0; i < nfail; ++i)
        fail_virt_buf[i] = fail_rank[i] == ORACLE_NO_RANK ? ORACLE_NO_RANK
                                                          : t->virt_of_phys[fail_rank[i]];
    s->fail_virt = fail_virt_buf;
    s->fail_round = fail_round;
    s->input = malloc((size_t)t->P * s->bytes);
    s->data = malloc((size_t)t->P * s->bytes);
    s->inbox = calloc(t->P, sizeof(inbox_t));
    s->has = calloc(t->P, 1);
    s->held = calloc((size_t)t->P, s->bytes);
    for (v = 0; v < t->P; ++v)
        memcpy(s->input + (size_t)v * s->bytes,
               (const unsigned char *)payload + (size_t)t->phys_of_virt[v] * s->bytes, s->bytes);
}

/* switch on the first and second failure-information scheme for this simulation */
static void sim_track_info(sim_t *s)
{
    const uint32_t P = s->t->P;
    s->track_info = 1;
    s->flcap = 2 * s->nfail + 4;
    s->fl = malloc(sizeof(uint32_t) * (size_t)P * s->flcap);
    s->fn = calloc(P, sizeof(uint32_t));
    s->fcount = calloc(P, sizeof(uint32_t));
    s->sel_ids = calloc(s->flcap, sizeof(uint32_t));
    s->ch_state = calloc(s->t->f + 1, sizeof(uint32_t));
    s->ch_count = calloc(s->t->f + 1, sizeof(uint32_t));
    s->ch_nids = calloc(s->t->f + 1, sizeof(uint32_t));
    s->ch_ids = calloc((size_t)(s->t->f + 1) * s->flcap, sizeof(uint32_t));
}

/* the selected message's failure information, ids as physical ranks; nids = ORACLE_NO_RANK if a list overflowed */
static void info_report(const sim_t *s, uint32_t nfail, uint32_t *info_count, uint32_t *info_nids, uint32_t *info_ids,
                        uint32_t *child /* [f+1][3 + nfail]: state, counter, list length, list; or NULL */)
{
    uint32_t i, c;
    for (i = 0; i < nfail; ++i) info_ids[i] = ORACLE_NO_RANK;
    *info_count = s->sel_count;
    *info_nids = s->info_overflow || s->sel_nids > nfail ? ORACLE_NO_RANK : s->sel_nids;
    for (i = 0; i < s->sel_nids && i < nfail; ++i) info_ids[i] = s->t->phys_of_virt[s->sel_ids[i]];
    if (!child) return;
    for (c = 0; c <= s->t->f; ++c) {
        uint32_t *row = child + (size_t)c * (3 + nfail);
        row[0] = s->ch_state[c];
        row[1] = s->ch_count[c];
        row[2] = s->ch_nids[c] > nfail ? ORACLE_NO_RANK : s->ch_nids[c];
        for (i = 0; i < nfail; ++i)
            row[3 + i] = i < s->ch_nids[c] ? s->t->phys_of_virt[s->ch_ids[(size_t)c * s->flcap + i]] : ORACLE_NO_RANK;
    }
}

static void sim_free(sim_t *s)
{
    free(s->input); free(s->data); free(s->inbox); free(s->has); free(s->held);
    free(s->trace_v); free(s->trace_sent); free(s->trace_flag); free(s->trace_msg);
    free(s->fl); free(s->fn); free(s->fcount); free(s->sel_ids);
    free(s->ch_state); free(s->ch_count); free(s->ch_nids); free(s->ch_ids);
    free(s->port_in); free(s->port_out);
    free(s->clock); free(s->finish);
    arena_release(s);
}

/* ------------------------------------------------------------------ */
/* entry points                                                         */

/* Structure of the tree and the groups for (P, f, root), all arrays indexed by
   PHYSICAL rank and holding physical ranks.  parent = -1 for the root;
   group = -1 for a process in no group; send_round = round of the tree-phase
   message (0 for the root).  Returns 0, or -1 for invalid arguments. */
int oracle_structure_shape(uint32_t P, uint32_t f, uint32_t root, int shape,
                           int64_t *parent, uint32_t *subtree, int64_t *group, uint32_t *gpos,
                           uint32_t *gsize, uint32_t *height, uint32_t *depth,
                           uint32_t *send_round, uint32_t *D_out)
{
    topo_t t;
    uint32_t v;
    if (topo_build(&t, P, f, root, shape) != 0) { topo_free(&t); return -1; }
    for (v = 0; v < P; ++v) {
        uint32_t p = t.phys_of_virt[v];
        parent[p] = t.parent[v] < 0 ? -1 : (int64_t)t.phys_of_virt[t.parent[v]];
        subtree[p] = t.subtree[v];
        group[p] = t.group[v];
        gpos[p] = t.gpos[v];
        gsize[p] = t.group[v] >= 0 ? t.gsize[t.group[v]] : 0;
        height[p] = t.height[v];
        depth[p] = t.depth[v];
        send_round[p] = v == 0 ? 0 : f + 1 + t.height[v];
    }
    *D_out = t.D;
    topo_free(&t);
    return 0;
}

int oracle_structure(uint32_t P, uint32_t f, uint32_t root,
                     int64_t *parent, uint32_t *subtree, int64_t *group, uint32_t *gpos,
                     uint32_t *gsize, uint32_t *height, uint32_t *depth,
                     uint32_t *send_round, uint32_t *D_out)
{
    return oracle_structure_shape(P, f, root, SHAPE_DEFAULT, parent, subtree, group, gpos, gsize, height, depth,
                                  send_round, D_out);
}

/* One reduce.  payload[P][elems] by physical rank.  Failure entries with rank
   ORACLE_NO_RANK are unused.  Outputs: result[elems] (valid when *status == OK),
   msgs[2] = {up-correction, tree} messages sent, *rounds = f + D.
   Optional traces (NULL to skip), indexed by physical rank: v_after_uc[P][elems]
   = value of each process after the up-correction phase; tree_sent/tree_flag[P]
   and tree_msg[P][elems] = whether, with which failed bit and with which value
   each process sent its tree message.  disable_uc != 0 skips the up-correction
   sends (control experiment: the plain tree).  Returns 0, -1 on bad arguments. */
static int reduce_impl(uint32_t P, uint32_t f, uint32_t elems, int dtype, int op, int disable_uc, int shape,
                       uint32_t *detected /* bit q = slot q of the failure list was detected as failed; or NULL */,
                       uint32_t root, const void *payload,
                       uint32_t nfail, const uint32_t *fail_rank, const uint32_t *fail_round,
                       void *result, uint32_t *status, uint64_t *msgs, uint32_t *rounds,
                       void *v_after_uc, uint8_t *tree_sent, uint8_t *tree_flag, void *tree_msg,
                       uint32_t *info_count, uint32_t *info_nids, uint32_t *info_ids, uint32_t *info_child)
{
    topo_t t;
    sim_t s;
    uint32_t *fv, v;
    int st;
    if (elems == 0 || (dtype == OR_F64 && op != OR_SUM) || dtype < 0 || dtype > 2) return -1;
    if (topo_build(&t, P, f, root, shape) != 0) { topo_free(&t); return -1; }
    *rounds = f + t.D;
    if (detected) *detected = 0;
    msgs[0] = msgs[1] = 0;
    if (info_count) {
        *info_count = *info_nids = 0;
        for (v = 0; v < nfail; ++v) info_ids[v] = ORACLE_NO_RANK;
        if (info_child) memset(info_child, 0, sizeof(uint32_t) * (f + 1) * (3 + nfail));
    }
    if (check_failures(P, nfail, fail_rank) != 0) {
        *status = OR_ST_BAD_FAILURE_SET;
        topo_free(&t);
        return 0;
    }
    fv = malloc(sizeof(uint32_t) * (nfail + 1));
    sim_init(&s, &t, elems, dtype, op, payload, nfail, fail_rank, fail_round, fv);
    s.disable_uc = disable_uc;
    if (info_count) sim_track_info(&s);
    if (v_after_uc) s.trace_v = calloc(P, s.bytes);
    if (tree_sent) s.trace_sent = calloc(P, 1);
    if (tree_flag) s.trace_flag = calloc(P, 1);
    if (tree_msg) s.trace_msg = calloc(P, s.bytes);
    memset(result, 0, s.bytes);
    st = run_reduce(&s, 0, result);
    if (st != OR_ST_OK) memset(result, 0, s.bytes);
    *status = (uint32_t)st;
    msgs[0] = s.sent[MSG_UC];
    msgs[1] = s.sent[MSG_TREE];
    if (detected) *detected = s.detected;
    if (info_count && st == OR_ST_OK) info_report(&s, nfail, info_count, info_nids, info_ids, info_child);
    for (v = 0; v < P; ++v) {
        uint32_t p = t.phys_of_virt[v];
        if (v_after_uc) memcpy((unsigned char *)v_after_uc + (size_t)p * s.bytes, s.trace_v + (size_t)v * s.bytes, s.bytes);
        if (tree_sent) tree_sent[p] = s.trace_sent[v];
        if (tree_flag) tree_flag[p] = s.trace_flag[v];
        if (tree_msg) memcpy((unsigned char *)tree_msg + (size_t)p * s.bytes, s.trace_msg + (size_t)v * s.bytes, s.bytes);
    }
    sim_free(&s);
    free(fv);
    topo_free(&t);
    return 0;
}

int oracle_reduce(uint32_t P, uint32_t f, uint32_t elems, int dtype, int op, int disable_uc,
                  uint32_t root, const void *payload,
                  uint32_t nfail, const uint32_t *fail_rank, const uint32_t *fail_round,
                  void *result, uint32_t *status, uint64_t *msgs, uint32_t *rounds,
                  void *v_after_uc, uint8_t *tree_sent, uint8_t *tree_flag, void *tree_msg)
{
    return reduce_impl(P, f, elems, dtype, op, disable_uc, SHAPE_DEFAULT, NULL, root, payload, nfail, fail_rank,
                       fail_round, result, status, msgs, rounds, v_after_uc, tree_sent, tree_flag, tree_msg, NULL, NULL,
                       NULL, NULL);
}

/* oracle_reduce for the tree shape `shape` (see topo_build), plus *detected (bit q = the process in slot q of the
   failure list was detected as failed, R8; may be NULL). */
int oracle_reduce_shape(uint32_t P, uint32_t f, uint32_t elems, int dtype, int op, int disable_uc, int shape,
                        uint32_t root, const void *payload,
                        uint32_t nfail, const uint32_t *fail_rank, const uint32_t *fail_round,
                        void *result, uint32_t *status, uint64_t *msgs, uint32_t *rounds, uint32_t *detected,
                        void *v_after_uc, uint8_t *tree_sent, uint8_t *tree_flag, void *tree_msg)
{
    return reduce_impl(P, f, elems, dtype, op, disable_uc, shape, detected, root, payload, nfail, fail_rank,
                       fail_round, result, status, msgs, rounds, v_after_uc, tree_sent, tree_flag, tree_msg, NULL, NULL,
                       NULL, NULL);
}

/* One reduce with the first and second failure-information scheme tracked
   (section "Failure information").  As oracle_reduce, plus: *info_count = the
   counter of the second scheme and info_ids[nfail] / *info_nids = the list of the
   first scheme (physical ranks, in the order appended, padded with
   ORACLE_NO_RANK) carried by the message the root selected; zeros / padding unless
   *status == OK.  *info_nids == ORACLE_NO_RANK reports a list that outgrew the
   number of listed failures (concatenated lists were not disjoint).
   info_child (may be NULL): [f+1][3 + nfail] words, for each child of the root in
   the order of the subtrees: state (0 no message, 1 message without the failed
   bit, 2 with it), counter, list length, list (physical ranks, padded). */
int oracle_reduce_info(uint32_t P, uint32_t f, uint32_t elems, int dtype, int op,
                       uint32_t root, const void *payload,
                       uint32_t nfail, const uint32_t *fail_rank, const uint32_t *fail_round,
                       void *result, uint32_t *status, uint64_t *msgs, uint32_t *rounds,
                       uint32_t *info_count, uint32_t *info_nids, uint32_t *info_ids, uint32_t *info_child)
{
    if (!info_count || !info_nids || !info_ids) return -1;
    return reduce_impl(P, f, elems, dtype, op, 0, SHAPE_DEFAULT, NULL, root, payload, nfail, fail_rank, fail_round,
                       result, status, msgs, rounds, NULL, NULL, NULL, NULL, info_count, info_nids, info_ids, info_child);
}

/* One allreduce.  Roots tried: physical ranks 0,1,..,f.  A failure listed for
   one of these ranks with fail_round != 0 is outside the semantics (the roots
   may fail only before the operation) => BAD_FAILURE_SET.  Global rounds keep
   counting over the attempts: attempt a occupies rounds a*2(f+D)+1 .. (a+1)*2(f+D).
   Outputs: result[elems]; has[P] (1 = the process holds the value at the end);
   out[P][elems] (the value held, zeros where has == 0; may be NULL);
   *attempts; msgs[4] = {up-correction, tree, broadcast tree, broadcast correction}
   summed over all attempts; *rounds = attempts * 2(f+D). */
static int allreduce_impl(uint32_t P, uint32_t f, uint32_t elems, int dtype, int op, int shape,
                          uint32_t *detected /* as in reduce_impl, over all attempts; or NULL */,
                          const void *payload,
                          uint32_t nfail, const uint32_t *fail_rank, const uint32_t *fail_round,
                          void *result, uint32_t *status, uint32_t *attempts, uint64_t *msgs,
                          uint32_t *rounds, uint8_t *has, void *out,
                          uint32_t *info_count, uint32_t *info_nids, uint32_t *info_ids, uint32_t *info_child)
{
    uint32_t a, i, v, base = 0;
    size_t bytes;
    uint32_t *fv;
    int st = OR_ST_NO_LIVE_ROOT;
    if (elems == 0 || (dtype == OR_F64 && op != OR_SUM) || dtype < 0 || dtype > 2) return -1;
    if (P < f + 2) return -1;
    bytes = elems * elem_size(dtype);
    memset(result, 0, bytes);
    memset(has, 0, P);
    if (out) memset(out, 0, (size_t)P * bytes);
    msgs[0] = msgs[1] = msgs[2] = msgs[3] = 0;
    *attempts = 0; *rounds = 0;
    if (detected) *detected = 0;
    if (shape < 1 || shape > 64) return -1;
    if (info_count) {
        *info_count = *info_nids = 0;
        for (i = 0; i < nfail; ++i) info_ids[i] = ORACLE_NO_RANK;
        if (info_child) memset(info_child, 0, sizeof(uint32_t) * (f + 1) * (3 + nfail));
    }
    if (check_failures(P, nfail, fail_rank) != 0) { *status = OR_ST_BAD_FAILURE_SET; return 0; }
    for (i = 0; i < nfail; ++i)
        if (fail_rank[i] != ORACLE_NO_RANK && fail_rank[i] <= f && fail_round[i] != 0) {
            *status = OR_ST_BAD_FAILURE_SET;
            return 0;
        }
    fv = malloc(sizeof(uint32_t) * (nfail + 1));
    for (a = 0; a <= f; ++a) {
        topo_t t;
        sim_t s;
        uint32_t Ra, n_alive = 0, n_ok = 0;
        int rst;
        topo_build(&t, P, f, a, shape);
        Ra = 2 * (f + t.D);
        sim_init(&s, &t, elems, dtype, op, payload, nfail, fail_rank, fail_round, fv);
        if (info_count) sim_track_info(&s);
        *attempts = a + 1;
        rst = run_reduce(&s, base, result);
        msgs[0] += s.sent[MSG_UC];
        msgs[1] += s.sent[MSG_TREE];
        if (rst == OR_ST_OK) {
            run_broadcast(&s, base + f + t.D, result);
            msgs[2] += s.sent[MSG_BCAST];
            msgs[3] += s.sent[MSG_BCORR];
        } else if (rst == OR_ST_ROOT_FAILED) {
            /* the rounds of the broadcast pass all the same: the failed root sends nothing, nobody comes to
               hold a value, and the root's children wait for its message in vain */
            run_broadcast(&s, base + f + t.D, result);
            memset(s.has, 0, P);
        } else {
            memset(s.has, 0, P);
        }
        if (detected) *detected |= s.detected;
        *rounds = base + Ra;
        /* "ok <- broadcast finished successfully", judged by every process that
           is still alive in the last round of the attempt */
        for (v = 0; v < P; ++v)
            if (alive(&s, v, base + Ra)) { ++n_alive; if (s.has[v]) ++n_ok; }
        if (rst == OR_ST_NO_CLEAN_SUBTREE) {
            st = OR_ST_NO_CLEAN_SUBTREE;
        } else if (n_ok == n_alive && n_alive > 0 && rst == OR_ST_OK) {
            st = OR_ST_OK;
            if (info_count) info_report(&s, nfail, info_count, info_nids, info_ids, info_child);   /* of the reduce that counted */
            for (v = 0; v < P; ++v) {
                uint32_t p = t.phys_of_virt[v];
                has[p] = s.has[v];
                if (out && s.has[v])
                    memcpy((unsigned char *)out + (size_t)p * bytes, s.held + (size_t)v * bytes, bytes);
            }
        } else if (n_ok == 0) {
            st = OR_ST_NO_LIVE_ROOT;      /* nobody got a value: try the successor */
        } else {
            st = OR_ST_INCONSISTENT;      /* some have it, some do not */
        }
        sim_free(&s);
        topo_free(&t);
        base += Ra;
        if (st != OR_ST_NO_LIVE_ROOT) break;
    }
    if (st != OR_ST_OK) memset(result, 0, bytes);
    *status = (uint32_t)st;
    free(fv);
    return 0;
}

int oracle_allreduce(uint32_t P, uint32_t f, uint32_t elems, int dtype, int op,
                     const void *payload,
                     uint32_t nfail, const uint32_t *fail_rank, const uint32_t *fail_round,
                     void *result, uint32_t *status, uint32_t *attempts, uint64_t *msgs,
                     uint32_t *rounds, uint8_t *has, void *out)
{
    return allreduce_impl(P, f, elems, dtype, op, SHAPE_DEFAULT, NULL, payload, nfail, fail_rank, fail_round, result,
                          status, attempts, msgs, rounds, has, out, NULL, NULL, NULL, NULL);
}

/* One allreduce with the failure information of oracle_reduce_info, taken from
   the reduce of the attempt whose result every survivor holds. */
int oracle_allreduce_info(uint32_t P, uint32_t f, uint32_t elems, int dtype, int op,
                          const void *payload,
                          uint32_t nfail, const uint32_t *fail_rank, const uint32_t *fail_round,
                          void *result, uint32_t *status, uint32_t *attempts, uint64_t *msgs,
                          uint32_t *rounds, uint8_t *has, void *out,
                          uint32_t *info_count, uint32_t *info_nids, uint32_t *info_ids, uint32_t *info_child)
{
    if (!info_count || !info_nids || !info_ids) return -1;
    return allreduce_impl(P, f, elems, dtype, op, SHAPE_DEFAULT, NULL, payload, nfail, fail_rank, fail_round, result,
                          status, attempts, msgs, rounds, has, out, info_count, info_nids, info_ids, info_child);
}

/* Batches: scenario i uses payload + i*payload_stride_bytes (stride 0 = one
   payload shared by all), root[i] (NULL = 0), failure rows i of [S][nfail].
   Scenarios are independent and are spread over `threads` OpenMP threads
   (<= 0: the runtime's default).  Returns the number of threads used, or -1. */
int oracle_reduce_batch(uint32_t P, uint32_t f, uint32_t elems, int dtype, int op,
                        uint32_t S, const uint32_t *root,
                        const void *payload, uint64_t payload_stride_bytes,
                        uint32_t nfail, const uint32_t *fail_rank, const uint32_t *fail_round,
                        void *result, uint32_t *status, uint64_t *msgs, int threads)
{
    int64_t i;
    int bad = 0, used = 1;
    size_t bytes = elems * elem_size(dtype);
#ifdef _OPENMP
    if (threads > 0) omp_set_num_threads(threads);
    used = omp_get_max_threads();
#endif
#pragma omp parallel for schedule(dynamic, 1)
    for (i = 0; i < (int64_t)S; ++i) {
        uint32_t rounds;
        int rc = oracle_reduce(P, f, elems, dtype, op, 0, root ? root[i] : 0,
                               (const unsigned char *)payload + (size_t)i * payload_stride_bytes,
                               nfail, fail_rank + (size_t)i * nfail, fail_round + (size_t)i * nfail,
                               (unsigned char *)result + (size_t)i * bytes, status + i,
                               msgs + 2 * (size_t)i, &rounds, NULL, NULL, NULL, NULL);
        if (rc != 0) {
#pragma omp atomic write
            bad = 1;
        }
    }
    return bad ? -1 : used;
}

int oracle_allreduce_batch(uint32_t P, uint32_t f, uint32_t elems, int dtype, int op,
                           uint32_t S, const void *payload, uint64_t payload_stride_bytes,
                           uint32_t nfail, const uint32_t *fail_rank, const uint32_t *fail_round,
                           void *result, uint32_t *status, uint32_t *attempts, uint64_t *msgs,
                           uint32_t *rounds, uint8_t *has /* [S][P] or NULL */,
                           void *out /* [S][P][elems] or NULL */, int threads)
{
    int64_t i;
    int bad = 0, used = 1;
    size_t bytes = elems * elem_size(dtype);
#ifdef _OPENMP
    if (threads > 0) omp_set_num_threads(threads);
    used = omp_get_max_threads();
#endif
#pragma omp parallel for schedule(dynamic, 1)
    for (i = 0; i < (int64_t)S; ++i) {
        uint8_t *h = has ? has + (size_t)i * P : malloc(P);
        int rc = oracle_allreduce(P, f, elems, dtype, op,
                                  (const unsigned char *)payload + (size_t)i * payload_stride_bytes,
                                  nfail, fail_rank + (size_t)i * nfail, fail_round + (size_t)i * nfail,
                                  (unsigned char *)result + (size_t)i * bytes, status + i,
                                  attempts + i, msgs + 4 * (size_t)i, rounds + i, h,
                                  out ? (unsigned char *)out + (size_t)i * P * bytes : NULL);
        if (!has) free(h);
        if (rc != 0) {
#pragma omp atomic write
            bad = 1;
        }
    }
    return bad ? -1 : used;
}

/* Batches of oracle_reduce_info / oracle_allreduce_info: info_count[S],
   info_nids[S], info_ids[S][nfail], info_child[S][f+1][3 + nfail] (or NULL). */
int oracle_reduce_info_batch(uint32_t P, uint32_t f, uint32_t elems, int dtype, int op,
                             uint32_t S, const uint32_t *root,
                             const void *payload, uint64_t payload_stride_bytes,
                             uint32_t nfail, const uint32_t *fail_rank, const uint32_t *fail_round,
                             void *result, uint32_t *status, uint64_t *msgs,
                             uint32_t *info_count, uint32_t *info_nids, uint32_t *info_ids,
                             uint32_t *info_child, int threads)
{
    int64_t i;
    int bad = 0, used = 1;
    size_t bytes = elems * elem_size(dtype);
#ifdef _OPENMP
    if (threads > 0) omp_set_num_threads(threads);
    used = omp_get_max_threads();
#endif
#pragma omp parallel for schedule(dynamic, 1)
    for (i = 0; i < (int64_t)S; ++i) {
        uint32_t rounds;
        int rc = oracle_reduce_info(P, f, elems, dtype, op, root ? root[i] : 0,
                                    (const unsigned char *)payload + (size_t)i * payload_stride_bytes,
                                    nfail, fail_rank + (size_t)i * nfail, fail_round + (size_t)i * nfail,
                                    (unsigned char *)result + (size_t)i * bytes, status + i,
                                    msgs + 2 * (size_t)i, &rounds,
                                    info_count + i, info_nids + i, info_ids + (size_t)i * nfail,
                                    info_child ? info_child + (size_t)i * (f + 1) * (3 + nfail) : NULL);
        if (rc != 0) {
#pragma omp atomic write
            bad = 1;
        }
    }
    return bad ? -1 : used;
}

int oracle_allreduce_info_batch(uint32_t P, uint32_t f, uint32_t elems, int dtype, int op,
                                uint32_t S, const void *payload, uint64_t payload_stride_bytes,
                                uint32_t nfail, const uint32_t *fail_rank, const uint32_t *fail_round,
                                void *result, uint32_t *status, uint32_t *attempts, uint64_t *msgs,
                                uint32_t *info_count, uint32_t *info_nids, uint32_t *info_ids,
                             uint32_t *info_child, int threads)
{
    int64_t i;
    int bad = 0, used = 1;
    size_t bytes = elems * elem_size(dtype);
#ifdef _OPENMP
    if (threads > 0) omp_set_num_threads(threads);
    used = omp_get_max_threads();
#endif
#pragma omp parallel for schedule(dynamic, 1)
    for (i = 0; i < (int64_t)S; ++i) {
        uint8_t *h = malloc(P);
        uint32_t rounds;
        int rc = oracle_allreduce_info(P, f, elems, dtype, op,
                                       (const unsigned char *)payload + (size_t)i * payload_stride_bytes,
                                       nfail, fail_rank + (size_t)i * nfail, fail_round + (size_t)i * nfail,
                                       (unsigned char *)result + (size_t)i * bytes, status + i,
                                       attempts + i, msgs + 4 * (size_t)i, &rounds, h, NULL,
                                       info_count + i, info_nids + i, info_ids + (size_t)i * nfail,
                                    info_child ? info_child + (size_t)i * (f + 1) * (3 + nfail) : NULL);
        free(h);
        if (rc != 0) {
#pragma omp atomic write
            bad = 1;
        }
    }
    return bad ? -1 : used;
}

/* ------------------------------------------------------------------ */
/* other tree shapes (R3) and the latency bookkeeping (R8)                */

/* Batches as oracle_reduce_batch / oracle_allreduce_batch for the tree shape `shape` (see topo_build), plus
   detected[S] (or NULL): bit q of detected[i] = the process in slot q of scenario i's failure list was detected
   as failed by a process that was alive (over all attempts of an allreduce). */
int oracle_reduce_shape_batch(uint32_t P, uint32_t f, uint32_t elems, int dtype, int op, int shape,
                              uint32_t S, const uint32_t *root,
                              const void *payload, uint64_t payload_stride_bytes,
                              uint32_t nfail, const uint32_t *fail_rank, const uint32_t *fail_round,
                              void *result, uint32_t *status, uint64_t *msgs, uint32_t *detected, int threads)
{
    int64_t i;
    int bad = 0, used = 1;
    size_t bytes = elems * elem_size(dtype);
#ifdef _OPENMP
    if (threads > 0) omp_set_num_threads(threads);
    used = omp_get_max_threads();
#endif
#pragma omp parallel for schedule(dynamic, 1)
    for (i = 0; i < (int64_t)S; ++i) {
        uint32_t rounds;
        int rc = reduce_impl(P, f, elems, dtype, op, 0, shape, detected ? detected + i : NULL, root ? root[i] : 0,
                             (const unsigned char *)payload + (size_t)i * payload_stride_bytes,
                             nfail, fail_rank + (size_t)i * nfail, fail_round + (size_t)i * nfail,
                             (unsigned char *)result + (size_t)i * bytes, status + i,
                             msgs + 2 * (size_t)i, &rounds, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL);
        if (rc != 0) {
#pragma omp atomic write
            bad = 1;
        }
    }
    return bad ? -1 : used;
}

int oracle_allreduce_shape_batch(uint32_t P, uint32_t f, uint32_t elems, int dtype, int op, int shape,
                                 uint32_t S, const void *payload, uint64_t payload_stride_bytes,
                                 uint32_t nfail, const uint32_t *fail_rank, const uint32_t *fail_round,
                                 void *result, uint32_t *status, uint32_t *attempts, uint64_t *msgs,
                                 uint32_t *rounds, uint8_t *has /* [S][P] or NULL */,
                                 void *out /* [S][P][elems] or NULL */, uint32_t *detected, int threads)
{
    int64_t i;
    int bad = 0, used = 1;
    size_t bytes = elems * elem_size(dtype);
#ifdef _OPENMP
    if (threads > 0) omp_set_num_threads(threads);
    used = omp_get_max_threads();
#endif
#pragma omp parallel for schedule(dynamic, 1)
    for (i = 0; i < (int64_t)S; ++i) {
        uint8_t *h = has ? has + (size_t)i * P : malloc(P);
        int rc = allreduce_impl(P, f, elems, dtype, op, shape, detected ? detected + i : NULL,
                                (const unsigned char *)payload + (size_t)i * payload_stride_bytes,
                                nfail, fail_rank + (size_t)i * nfail, fail_round + (size_t)i * nfail,
                                (unsigned char *)result + (size_t)i * bytes, status + i,
                                attempts + i, msgs + 4 * (size_t)i, rounds + i, h,
                                out ? (unsigned char *)out + (size_t)i * P * bytes : NULL, NULL, NULL, NULL, NULL);
        if (!has) free(h);
        if (rc != 0) {
#pragma omp atomic write
            bad = 1;
        }
    }
    return bad ? -1 : used;
}

/* Event-driven times of the reduce (R9), a batch: as oracle_reduce_shape_batch, plus t_done[S] = the moment the
   root delivers (with status NO_CLEAN_SUBTREE: the moment it has gone through all its children; ORACLE_NEVER
   when the root has failed or the failure set is bad) and t_proc[S][P] (may be NULL; by physical rank) = the
   moment each process has done its part (sent to its parent; the root: t_done), ORACLE_NEVER for a process that
   stops before.  t_msg, t_timeout >= 1. */
int oracle_reduce_timed_batch(uint32_t P, uint32_t f, uint32_t elems, int dtype, int op, int shape,
                              uint32_t S, const uint32_t *root,
                              const void *payload, uint64_t payload_stride_bytes,
                              uint32_t nfail, const uint32_t *fail_rank, const uint32_t *fail_round,
                              uint64_t t_msg, uint64_t t_timeout,
                              void *result, uint32_t *status, uint64_t *msgs, uint64_t *t_done, uint64_t *t_proc,
                              int threads)
{
    int64_t i;
    int bad = 0, used = 1;
    size_t bytes = elems * elem_size(dtype);
    if (t_msg == 0 || t_timeout == 0 || elems == 0 || (dtype == OR_F64 && op != OR_SUM) || dtype < 0 || dtype > 2)
        return -1;
#ifdef _OPENMP
    if (threads > 0) omp_set_num_threads(threads);
    used = omp_get_max_threads();
#endif
#pragma omp parallel for schedule(dynamic, 1)
    for (i = 0; i < (int64_t)S; ++i) {
        topo_t t;
        sim_t s;
        uint32_t *fv, v;
        int st;
        const uint32_t *fr = fail_rank + (size_t)i * nfail, *fo = fail_round + (size_t)i * nfail;
        unsigned char *res = (unsigned char *)result + (size_t)i * bytes;
        memset(res, 0, bytes);
        msgs[2 * i] = msgs[2 * i + 1] = 0;
        t_done[i] = ORACLE_NEVER;
        if (t_proc) for (v = 0; v < P; ++v) t_proc[(size_t)i * P + v] = ORACLE_NEVER;
        if (topo_build(&t, P, f, root ? root[i] : 0, shape) != 0) {
            topo_free(&t);
#pragma omp atomic write
            bad = 1;
            continue;
        }
        if (check_failures(P, nfail, fr) != 0) {
            status[i] = OR_ST_BAD_FAILURE_SET;
            topo_free(&t);
            continue;
        }
        fv = malloc(sizeof(uint32_t) * (nfail + 1));
        sim_init(&s, &t, elems, dtype, op, (const unsigned char *)payload + (size_t)i * payload_stride_bytes,
                 nfail, fr, fo, fv);
        s.timed = 1;
        s.t_msg = t_msg;
        s.t_timeout = t_timeout;
        s.clock = calloc(P, sizeof(uint64_t));
        s.finish = malloc(sizeof(uint64_t) * P);
        for (v = 0; v < P; ++v) s.finish[v] = ORACLE_NEVER;
        s.t_done = ORACLE_NEVER;
        st = run_reduce(&s, 0, res);
        if (st != OR_ST_OK) memset(res, 0, bytes);
        status[i] = (uint32_t)st;
        msgs[2 * i] = s.sent[MSG_UC];
        msgs[2 * i + 1] = s.sent[MSG_TREE];
        t_done[i] = s.t_done;
        if (t_proc) for (v = 0; v < P; ++v) t_proc[(size_t)i * P + t.phys_of_virt[v]] = s.finish[v];
        sim_free(&s);
        free(fv);
        topo_free(&t);
    }
    return bad ? -1 : used;
}

/* Message steps of one failure-free attempt with root 0 (R8): steps[4] = per kind of message (up-correction,
   tree, broadcast down the tree, broadcast correction) the sum over its rounds of the number of messages the
   busiest process sends or receives in the round.  Counted from a failure-free run of the simulation with one
   value per process.  Returns 0, -1 for invalid arguments. */
int oracle_latency_steps(uint32_t P, uint32_t f, int shape, uint32_t *steps)
{
    topo_t t;
    sim_t s;
    uint32_t none = ORACLE_NO_RANK, zero = 0, fv[2];
    uint64_t *payload, result = 0;
    int k;
    if (topo_build(&t, P, f, 0, shape) != 0) { topo_free(&t); return -1; }
    payload = calloc(P, sizeof(uint64_t));
    sim_init(&s, &t, 1, OR_I64, OR_SUM, payload, 1, &none, &zero, fv);
    s.count_steps = 1;
    s.port_in = calloc(P, sizeof(uint32_t));
    s.port_out = calloc(P, sizeof(uint32_t));
    run_reduce(&s, 0, &result);
    run_broadcast(&s, f + t.D, &result);
    for (k = 0; k < 4; ++k) steps[k] = s.steps[k];
    sim_free(&s);
    free(payload);
    topo_free(&t);
    return 0;
}

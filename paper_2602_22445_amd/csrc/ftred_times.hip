// Event-driven times of the reduce (entry point ftred_reduce_times).
//
// The paper's processes run by themselves: the active phase is a property of a
// process, not of the system (section "Related work", last paragraph), a receive
// from a failed sender ends by a time-out and the failure monitor's confirmation
// and is retried while the monitor says the sender lives (section "Up-Correction",
// last paragraph; liveness part of the proof in "Reduce / Properties").  The model
// of this library: every process starts at time 0 with a clock of its own; a send
// takes t_msg of the sender's time and the message is at the receiver when the
// send ends; a receive ends at once if the message is there, at its arrival
// otherwise; if the sender has stopped without sending, the receiver asks the
// monitor after every t_timeout of waiting and gives up at the first such moment
// that lies after the moment the sender stopped.  What is sent and received is
// what the round model sends and receives (a process awaits named senders in a
// fixed order), so values, statuses and counters are those of ftred_run_reduce;
// here only the clocks are worked out, from the failure lists alone.
//
// Two launches.  The first writes, for every process, the time it is done when
// nobody fails: t_msg x (f + 1 + its height), where a short last group (fewer
// exchange rounds than f) counts as absent, because its members' messages are at
// their parents before those have ended their own exchange.  The second, one
// wavefront per scenario, redoes what the failures touch: a process's time differs
// from that only if its group or the group of somebody below it holds a listed
// process, so the members of the listed processes' groups and their ancestors are
// worked out level by level from the deepest: the clock after the exchange in the
// up-correction group (Algorithm "Up-correction": send, then receive, round by
// round), the children's entries (a time with the failed bit of the message, or
// the moment the child stopped), the send.  Last the root: children in order
// until a message without the failed bit is there (Algorithm "reduce at the
// root").
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>

#include "../../include/ftred.h"
#include "ftred_geom.h"
#include "ftred_kernels.h"
#include "ftred_plan.h"

namespace ftred {
namespace {

constexpr unsigned long long kNever = ~0ull;
constexpr unsigned long long kStopped = 1ull << 63;      // working entry of a process that has stopped: low bits = when
constexpr unsigned long long kFailedBit = 1ull << 62;    // working entry of a sender: its message carries the failed bit
constexpr unsigned long long kTimeMask = kFailedBit - 1ull;

constexpr uint32_t kFillChunk = 4096;    // entries one workgroup of the first launch writes

struct TimeArgs {
    Geom g;
    const uint32_t* root;          // [S] or nullptr
    const uint32_t* fail_rank;
    const uint32_t* fail_round;
    unsigned long long t_msg, t_timeout;
    unsigned long long* t_done;    // [S]
    unsigned long long* t_proc;    // [S][P] by physical rank
    uint32_t S;
};


// the receiver's clock when it gives up on a sender that stopped at `stopped`: the first moment own + k * tau
// (k >= 1) that lies after it
__device__ __forceinline__ unsigned long long give_up(unsigned long long own, unsigned long long stopped,
                                                      unsigned long long tau)
{
    unsigned long long k = 1;
    if (stopped >= own + tau) k = (stopped - own) / tau + 1ull;
    return own + k * tau;
}

// Clock of member `me` of row j's up-correction group (gs members) after the exchange; the clocks of all members
// are worked out, since a member's waits depend on the others' clocks (Algorithm "Up-correction": in round t send
// to the target, then receive from the source).  The arrays are indexed by member numbers known at run time only
// and live in private memory; LDS for them (20 KiB per wavefront) was measured slower on large batches.
__device__ unsigned long long exchange_clock(const Geom& g, const FailTab& ft, uint32_t j, uint32_t gs, uint32_t me,
                                             unsigned long long m, unsigned long long tau)
{
    uint32_t lim[16];              // exchange rounds in which member w takes part
    unsigned long long clock[16], stamp[16];
    for (uint32_t w = 0; w < 16u; ++w) { lim[w] = gs; clock[w] = 0; }
    for (uint32_t q = 0; q < ft.n; ++q)
        if (ft.row[q] == j) lim[ft.idx[q] & 15u] = ft.uc[q];
    const uint32_t rounds = g.f < gs - 1u ? g.f : gs - 1u;
    for (uint32_t t = 1; t <= rounds; ++t) {
        for (uint32_t w = 0; w < gs; ++w) {
            if (t <= lim[w]) clock[w] += m;
            stamp[w] = clock[w];
        }
        for (uint32_t w = 0; w < gs; ++w) {
            if (t > lim[w]) continue;
            const uint32_t src = exchange_source(w, t, gs);
            if (t <= lim[src]) clock[w] = clock[w] > stamp[src] ? clock[w] : stamp[src];
            else clock[w] = give_up(clock[w], clock[src], tau);      // src has stopped: its clock stands
        }
    }
    return clock[me & 15u];
}

// is the scenario's failure set one the semantics cover (ranks below P, no rank twice, root below P)?
__device__ bool bad_failure_set(const Geom& g, const uint32_t* fr, uint32_t root)
{
    bool bad = root >= g.P;
    for (uint32_t q = 0; q < g.f; ++q) {
        if (fr[q] == kNoRank) continue;
        if (fr[q] >= g.P) bad = true;
        for (uint32_t q2 = 0; q2 < q; ++q2) bad = bad || fr[q2] == fr[q];
    }
    return bad;
}

// Working entries are read and written past the first-level cache: lanes of the wavefront hand them to each other
// through memory between two barriers.
__device__ __forceinline__ unsigned long long ld_entry(const unsigned long long* p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_entry(unsigned long long* p, unsigned long long v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// The parent's clock after it has dealt with one child (working entry `raw`), and the failed bit it passes on.
__device__ __forceinline__ void take_child(unsigned long long raw, unsigned long long tau, unsigned long long& clock,
                                           bool& flag, bool& present)
{
    present = (raw & kStopped) == 0ull;
    if (present) {
        const unsigned long long t = raw & kTimeMask;
        clock = clock > t ? clock : t;
        flag = flag || (raw & kFailedBit) != 0ull;
    } else {
        clock = give_up(clock, raw & kTimeMask, tau);
        flag = true;
    }
}

// Working entry of the process at position j of subtree i: its clock after the exchange, its children in ascending
// order, its send (Algorithm "reduce at non-roots").  A process that has stopped by its send round waits for nobody:
// its clock stands where the exchange left it.
__device__ unsigned long long node_entry(const TimeArgs& A, const FailTab& ft, const unsigned long long* tp, uint32_t root,
                                         uint32_t j, uint32_t i)
{
    const Geom& g = A.g;
    const uint32_t gs = group_size(g, j);
    bool listed_row = false, sends = true;
    for (uint32_t q = 0; q < ft.n; ++q)
        if (ft.row[q] == j) {
            listed_row = true;
            if (ft.idx[q] == i) sends = ft.tree[q] != 0u;
        }
    unsigned long long clock;
    if (!listed_row) {
        clock = (unsigned long long)(g.f < gs - 1u ? g.f : gs - 1u) * A.t_msg;
    } else {
        clock = exchange_clock(g, ft, j, gs, i, A.t_msg, A.t_timeout);
    }
    if (!sends) return clock | kStopped;
    bool flag = false;
    sh_for_children(g, subtree_size(g, i), j, [&](uint32_t jc) {
        bool present;
        take_child(ld_entry(tp + relabel(1u + jc * g.W + i, root)), A.t_timeout, clock, flag, present);
    });
    return (clock + A.t_msg) | (flag ? kFailedBit : 0ull);
}

// Every process's time when nobody fails (a failure set outside the semantics: "never").
__global__ void __launch_bounds__(256) times_fill_kernel(TimeArgs A, uint32_t blocks_per_scen, FastDiv div_bps)
{
    __shared__ uint32_t s_bad;
    const Geom& g = A.g;
    const uint32_t s = fdiv(blockIdx.x, div_bps);
    const uint32_t b = blockIdx.x - s * blocks_per_scen;
    const uint32_t root = A.root ? A.root[s] : 0u;
    const uint32_t F = g.f > 0 ? g.f : 1u;
    if (threadIdx.x == 0) s_bad = bad_failure_set(g, A.fail_rank + size_t(s) * F, root) ? 1u : 0u;
    __syncthreads();
    // a workgroup writes kFillChunk consecutive entries (a few KiB of work per look at the failure list)
    for (uint32_t p = b * kFillChunk + threadIdx.x; p < g.P && p < (b + 1u) * kFillChunk; p += 256u) {
        unsigned long long* own = A.t_proc + size_t(s) * g.P + p;
        if (s_bad) { *own = kNever; continue; }
        const uint32_t v = relabel(p, root);
        if (v == 0) continue;                                // the root: the second launch
        const uint32_t j = fdiv(v - 1u, g.divW), i = v - 1u - j * g.W;
        unsigned long long rounds;
        if (j == g.M - 1u) {
            // the deepest position of its subtree: its exchange (shorter in a short group), its send
            const uint32_t gs = group_size(g, j);
            rounds = (g.f < gs - 1u ? g.f : gs - 1u) + 1u;
        } else {
            // f exchange rounds, then a send one t_msg after the last child's; a member of a short last group
            // sends no later than its parent ends its exchange, so for heights it is not there
            uint32_t m = subtree_size(g, i);
            if (group_size(g, g.M - 1u) <= g.f && i < g.nlast) m -= 1u;
            uint32_t h;
            if (g.shape == kShapeBinary) {
                // the largest h with (j + 1) 2^h <= m
                h = ilog2(m) - ilog2(j + 1u);
                if (((j + 1u) << h) > m) --h;
            } else {
                h = sh_height_m(g.shape, m, j);
            }
            rounds = g.f + 1u + h;
        }
        *own = rounds * A.t_msg;
    }
}

// What the failures of one scenario touch, by one wavefront.
__global__ void __launch_bounds__(64) times_fix_kernel(TimeArgs A)
{
    __shared__ FailTab ft;
    __shared__ uint32_t seed_j[256], seed_i[256];
    __shared__ uint32_t nseeds;
    const Geom& g = A.g;
    const uint32_t s = blockIdx.x, lane = threadIdx.x;
    const uint32_t root = A.root ? A.root[s] : 0u;
    const uint32_t F = g.f > 0 ? g.f : 1u;
    unsigned long long* tp = A.t_proc + size_t(s) * g.P;
    if (bad_failure_set(g, A.fail_rank + size_t(s) * F, root)) {      // the same answer in every lane
        if (lane == 0) A.t_done[s] = kNever;
        return;
    }
    load_failtab(ft, g, A.fail_rank, A.fail_round, s, root, 0u);
    __syncthreads();
    // the members of every group that holds a listed process (the root is no tree member: it comes last)
    if (lane == 0) {
        uint32_t n = 0;
        for (uint32_t q = 0; q < ft.n; ++q) {
            const uint32_t j = ft.row[q];
            if (ft.vr[q] == kNoRank || j == kNoRank) continue;
            bool seen = false;
            for (uint32_t q2 = 0; q2 < q; ++q2) seen = seen || (ft.vr[q2] != kNoRank && ft.row[q2] == j);
            if (seen) continue;
            for (uint32_t i = 0; i < row_members(g, j); ++i) { seed_j[n] = j; seed_i[n] = i; ++n; }
        }
        nseeds = n;
    }
    __syncthreads();
    const uint32_t n = nseeds;
    // them and their ancestors, the deepest first: a level reads what the one below has left
    for (uint32_t d = n > 0u ? g.D : 0u; d >= 1u; --d) {
        for (uint32_t k = lane; k < n; k += 64u) {
            uint32_t j = seed_j[k];
            const uint32_t i = seed_i[k];
            uint32_t dj = sh_depth(g, j);
            if (dj < d) continue;
            for (; dj > d; --dj) j = sh_parent(g, j);
            st_entry(tp + relabel(1u + j * g.W + i, root), node_entry(A, ft, tp, root, j, i));
        }
        __syncthreads();
    }
    if (lane == 0) {
        // the root's exchange: member a-1 of the last group, if it is in one (section "Up-Correction")
        unsigned long long clock = 0;
        if (g.a > 1) clock = exchange_clock(g, ft, g.M - 1u, g.a, g.a - 1u, A.t_msg, A.t_timeout);
        // its children in order until a message without the failed bit is there (Algorithm "reduce at the root")
        bool waits = ft.root_alive != 0u;
        for (uint32_t k = 0; k < g.W && waits; ++k) {
            bool flag = false, present;
            take_child(ld_entry(tp + relabel(1u + k, root)), A.t_timeout, clock, flag, present);
            if (present && !flag) waits = false;
        }
        const unsigned long long done = ft.root_alive ? clock : kNever;
        A.t_done[s] = done;
        tp[root] = done;
    }
    __syncthreads();
    // working entries into their final form: a time, or "never" for a process that stopped; four ancestors at a
    // time, so that their loads are in flight together
    for (uint32_t k = lane; k < n; k += 64u) {
        uint32_t j = seed_j[k];
        const uint32_t i = seed_i[k];
        bool more = true;
        while (more) {
            unsigned long long* e[4];
            unsigned long long raw[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                e[u] = more ? tp + relabel(1u + j * g.W + i, root) : nullptr;
                if (more && j == 0) more = false;
                else if (more) j = sh_parent(g, j);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) raw[u] = e[u] ? ld_entry(e[u]) : 0ull;
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (e[u]) st_entry(e[u], (raw[u] & kStopped) ? kNever : (raw[u] & kTimeMask));
        }
    }
}

}  // namespace
}  // namespace ftred

using namespace ftred;

extern "C" int ftred_reduce_times(const ftred_plan_t* plan, uint32_t S, const uint32_t* root, const uint32_t* fail_rank,
                                  const uint32_t* fail_round, uint64_t t_msg, uint64_t t_timeout, uint64_t* t_done,
                                  uint64_t* t_proc, void* hip_stream)
{
    if (!plan) return set_error(FTRED_EINVAL, "ftred_reduce_times: plan is NULL");
    if (S == 0) return set_error(FTRED_EINVAL, "ftred_reduce_times: S must be >= 1");
    if (!fail_rank || !fail_round || !t_done || !t_proc)
        return set_error(FTRED_EINVAL, "ftred_reduce_times: fail_rank, fail_round, t_done and t_proc are required");
    if (t_msg == 0 || t_timeout == 0 || t_msg >= (uint64_t(1) << 32) || t_timeout >= (uint64_t(1) << 32))
        return set_error(FTRED_EINVAL, "ftred_reduce_times: t_msg and t_timeout must lie in 1 .. 2^32 - 1");
    const Geom& g = plan->g;
    hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
    TimeArgs A;
    memset(&A, 0, sizeof(A));
    A.g = g;
    A.root = root;
    A.fail_rank = fail_rank;
    A.fail_round = fail_round;
    A.t_msg = t_msg;
    A.t_timeout = t_timeout;
    A.t_done = reinterpret_cast<unsigned long long*>(t_done);
    A.t_proc = reinterpret_cast<unsigned long long*>(t_proc);
    A.S = S;
    const uint32_t bps = (g.P + kFillChunk - 1u) / kFillChunk;
    if (uint64_t(S) * bps >= (uint64_t(1) << 31))
        return set_error(FTRED_EUNSUPPORTED, "ftred_reduce_times: S = %u scenarios need too many workgroups; split the batch", S);
    hipLaunchKernelGGL(times_fill_kernel, dim3(S * bps), dim3(256), 0, st, A, bps, make_fastdiv(bps));
    HIP_TRY(hipGetLastError());
    hipLaunchKernelGGL(times_fix_kernel, dim3(S), dim3(64), 0, st, A);
    HIP_TRY(hipGetLastError());
    return FTRED_OK;
}

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
// One launch per depth of the tree, deepest first; one thread per process.  A
// thread works out its clock after the exchange in its up-correction group
// (Algorithm "Up-correction": send, then receive, round by round; closed form
// where nobody of the group is listed), takes its children's entries from t_proc,
// where an earlier launch left them (a time with the failed bit of the message,
// or the moment the child stopped), waits for each child in order, sends, and
// leaves its own entry; it rewrites its children's entries in their final form.
// A last launch is the root: children in order until a message without the
// failed bit is there (Algorithm "reduce at the root").
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

struct TimeLevel {
    uint32_t depth, j_lo, j_hi, filter;
    uint32_t blocks_per_scen;
    FastDiv div_bps;
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

// Clocks of the members of row j's up-correction group (gs members) after the exchange, all of them: a member's
// waits depend on the others' clocks.
__device__ void exchange_clocks(const Geom& g, const FailTab& ft, uint32_t j, uint32_t gs, unsigned long long m,
                                unsigned long long tau, unsigned long long* clock /* [16] */)
{
    uint32_t lim[16];              // exchange rounds in which member w takes part
    unsigned long long stamp[16];
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

// Takes the working entry of a child, advances the parent's clock (if it waits for it at all) and leaves the
// child's entry in its final form.
__device__ __forceinline__ void take_child(unsigned long long* cp, bool waits, unsigned long long tau,
                                           unsigned long long& clock, bool& flag, bool& present)
{
    const unsigned long long raw = *cp;
    present = (raw & kStopped) == 0ull;
    if (present) {
        const unsigned long long t = raw & kTimeMask;
        if (waits) {
            clock = clock > t ? clock : t;
            flag = flag || (raw & kFailedBit) != 0ull;
        }
        *cp = t;
    } else {
        if (waits) {
            clock = give_up(clock, raw & kTimeMask, tau);
            flag = true;
        }
        *cp = kNever;
    }
}

__global__ void __launch_bounds__(256) times_level_kernel(TimeArgs A, TimeLevel lv)
{
    __shared__ FailTab ft;
    __shared__ uint32_t s_bad;
    const Geom& g = A.g;
    const uint32_t tid = threadIdx.x;
    const uint32_t s = fdiv(blockIdx.x, lv.div_bps);
    const uint32_t b = blockIdx.x - s * lv.blocks_per_scen;
    const uint32_t root = A.root ? A.root[s] : 0u;
    const uint32_t F = g.f > 0 ? g.f : 1u;
    load_failtab(ft, g, A.fail_rank, A.fail_round, s, root, 0u);
    if (tid == 64) s_bad = bad_failure_set(g, A.fail_rank + size_t(s) * F, root) ? 1u : 0u;
    __syncthreads();

    const uint32_t W = g.W;
    const uint32_t it = b * 256u + tid;
    const uint32_t r = fdiv(it, g.divW);
    const uint32_t i = it - r * W;
    const uint32_t j = lv.j_lo + r;
    if (j >= lv.j_hi || (lv.filter && sh_depth(g, j) != lv.depth) || i >= row_members(g, j)) return;
    unsigned long long* tp = A.t_proc + size_t(s) * g.P;
    unsigned long long* own = tp + relabel(1u + j * W + i, root);
    if (s_bad) { *own = kNever; return; }

    // the exchange in the up-correction group
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
        unsigned long long ck[16];
        exchange_clocks(g, ft, j, gs, A.t_msg, A.t_timeout, ck);
        clock = ck[i & 15u];
    }
    // the children in order, then the send to the parent (Algorithm "reduce at non-roots"); a process that has
    // stopped by its send round waits for nobody, and its clock stands where the exchange left it
    bool flag = false;
    sh_for_children(g, subtree_size(g, i), j, [&](uint32_t jc) {
        bool present;
        take_child(tp + relabel(1u + jc * W + i, root), sends, A.t_timeout, clock, flag, present);
    });
    if (sends) *own = (clock + A.t_msg) | (flag ? kFailedBit : 0ull);
    else *own = clock | kStopped;
}

__global__ void __launch_bounds__(64) times_root_kernel(TimeArgs A)
{
    __shared__ FailTab ft;
    const Geom& g = A.g;
    const uint32_t s = blockIdx.x;
    const uint32_t root = A.root ? A.root[s] : 0u;
    const uint32_t F = g.f > 0 ? g.f : 1u;
    load_failtab(ft, g, A.fail_rank, A.fail_round, s, root, 0u);
    __syncthreads();
    if (threadIdx.x != 0) return;
    unsigned long long* tp = A.t_proc + size_t(s) * g.P;
    if (bad_failure_set(g, A.fail_rank + size_t(s) * F, root)) {
        // the level launches have left "never" for every process with a place in the tree; the one left is the
        // root, or process 0 if the root is no process at all
        A.t_done[s] = kNever;
        tp[root < g.P ? root : 0u] = kNever;
        return;
    }
    // the root's exchange: member a-1 of the short last group, if it is in one (section "Up-Correction")
    unsigned long long clock = 0;
    if (g.a > 1) {
        unsigned long long ck[16];
        exchange_clocks(g, ft, g.M - 1u, g.a, A.t_msg, A.t_timeout, ck);
        clock = ck[(g.a - 1u) & 15u];
    }
    // its children in order until a message without the failed bit is there (Algorithm "reduce at the root"); a
    // root that has stopped waits for nobody
    bool waits = ft.root_alive != 0u;
    for (uint32_t k = 0; k < g.W; ++k) {
        bool flag = false, present;
        take_child(tp + relabel(1u + k, root), waits, A.t_timeout, clock, flag, present);
        if (waits && present && !flag) waits = false;
    }
    const unsigned long long done = ft.root_alive ? clock : kNever;
    A.t_done[s] = done;
    tp[root] = done;
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
    for (uint32_t d = g.D; d >= 1; --d) {           // the rows of a subtree have depths 1 .. D
        TimeLevel lv;
        memset(&lv, 0, sizeof(lv));
        lv.depth = d;
        if (g.shape == kShapeBinomial) {
            // depth = 1 + number of one bits of the position: no range; the first such position is 2^(d-1) - 1
            lv.j_lo = d > 32u ? g.M : uint32_t((uint64_t(1) << (d - 1u)) - 1u);
            lv.j_hi = g.M;
            lv.filter = 1;
        } else {
            // level d-1 of a k-ary heap: positions (k^(d-1) - 1) / (k - 1) .. + k^(d-1) - 1
            uint64_t first = 0, count = 1;
            for (uint32_t l = 1; l < d && first < g.M; ++l) { first += count; count *= g.shape; }
            lv.j_lo = first < g.M ? uint32_t(first) : g.M;
            lv.j_hi = first + count < g.M ? uint32_t(first + count) : g.M;
        }
        if (lv.j_lo >= lv.j_hi) continue;
        const uint64_t items = uint64_t(lv.j_hi - lv.j_lo) * g.W;
        lv.blocks_per_scen = uint32_t((items + 255u) / 256u);
        lv.div_bps = make_fastdiv(lv.blocks_per_scen);
        if (uint64_t(S) * lv.blocks_per_scen >= (uint64_t(1) << 31))
            return set_error(FTRED_EUNSUPPORTED, "ftred_reduce_times: S = %u scenarios need too many workgroups; split the batch", S);
        hipLaunchKernelGGL(times_level_kernel, dim3(S * lv.blocks_per_scen), dim3(256), 0, st, A, lv);
        HIP_TRY(hipGetLastError());
    }
    hipLaunchKernelGGL(times_root_kernel, dim3(S), dim3(64), 0, st, A);
    HIP_TRY(hipGetLastError());
    return FTRED_OK;
}

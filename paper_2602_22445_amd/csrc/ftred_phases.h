// Kernels that do not depend on the reduction's arithmetic: scenario check,
// and the broadcast half of the allreduce (tree-down and correction rounds);
// plus the per-process index arithmetic shared by host and device.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ftred_geom.h"
#include "ftred_kernels.h"
#include "ftred_wave.h"

namespace ftred {

// ---------------------------------------------------------------------------
// partners of one process (physical ranks in, physical ranks out)

struct PartnerInfo {
    uint32_t parent, n_children, children[32];      // the root has f+1 children, a process of a binomial tree up to 32
    uint32_t group_id, group_size, group_pos, group[16];
    uint32_t subtree, depth, height, send_round;
};

FT_HD void partners_of(const Geom& g, uint32_t root, uint32_t rank, PartnerInfo& o)
{
    const uint32_t v = relabel(rank, root);
    o.n_children = 0;
    o.group_id = kNoRank;
    o.group_size = 0;
    o.group_pos = 0;
    if (v == 0) {
        // the root: f+1 children, the processes numbered 1..f+1
        o.parent = kNoRank;
        for (uint32_t i = 0; i < g.W; ++i) o.children[o.n_children++] = relabel(1 + i, root);
        o.subtree = 0; o.depth = 0; o.height = g.D; o.send_round = 0;
        if (g.a > 1) {       // member a-1 of the short last group
            o.group_id = g.M - 1;
            for (uint32_t i = 0; i + 1 < g.a; ++i) o.group[i] = relabel(1 + (g.M - 1) * g.W + i, root);
            o.group[g.a - 1] = rank;
            o.group_size = g.a;
            o.group_pos = g.a - 1;
        }
        return;
    }
    const uint32_t j = fdiv(v - 1, g.divW);
    const uint32_t i = v - 1 - j * g.W;
    o.parent = j == 0 ? relabel(0, root) : relabel(1 + sh_parent(g, j) * g.W + i, root);
    sh_for_children(g, subtree_size(g, i), j, [&](uint32_t jc) {
        if (o.n_children < 32u) o.children[o.n_children++] = relabel(1 + jc * g.W + i, root);
    });
    o.subtree = i + 1;
    o.depth = sh_depth(g, j);
    o.height = sh_height(g, i, j);
    o.send_round = g.f + 1 + o.height;
    o.group_id = j;
    const uint32_t nk = row_members(g, j);
    for (uint32_t k = 0; k < nk; ++k) o.group[k] = relabel(1 + j * g.W + k, root);
    o.group_size = nk;
    if (j == g.M - 1 && g.a > 1) {
        o.group[nk] = relabel(0, root);
        o.group_size = g.a;
    }
    o.group_pos = i;
}

// ---------------------------------------------------------------------------
// scenario check: one thread per scenario

__global__ void zero_words_kernel(uint32_t* p, uint32_t n)
{
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

__global__ void fill_words_kernel(uint32_t* p, size_t n, uint32_t value)
{
    const size_t i = size_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i < n) p[i] = value;
}

__global__ void prepass_kernel(Geom g, uint32_t kind /* 0 reduce, 1 allreduce */, uint32_t S, const uint32_t* root,
                               const uint32_t* fail_rank, const uint32_t* fail_round, uint32_t* status,
                               uint32_t* attempts, unsigned long long* msgs, uint32_t nmsg, unsigned char* result,
                               uint32_t* retry_list, uint32_t* retry_count)
{
    const uint32_t s = blockIdx.x * blockDim.x + threadIdx.x;
    if (s >= S) return;
    const uint32_t F = g.f > 0 ? g.f : 1;
    bool bad = false;
    uint32_t lead = 0;        // bit c: root candidate c failed before the operation
    for (uint32_t q = 0; q < F; ++q) {
        const uint32_t r = fail_rank[size_t(s) * F + q];
        if (r == kNoRank) continue;
        if (q >= g.f || r >= g.P) { bad = true; continue; }
        for (uint32_t q2 = 0; q2 < q; ++q2)
            if (fail_rank[size_t(s) * F + q2] == r) bad = true;
        if (kind == 1 && r <= g.f) {
            if (fail_round[size_t(s) * F + q] != 0) bad = true; else lead |= 1u << r;
        }
    }
    if (root && root[s] >= g.P) bad = true;
    uint32_t a = 0;
    while ((lead >> a) & 1u) ++a;
    status[s] = bad ? kStBadFailureSet : kStOk;
    if (attempts) attempts[s] = bad ? 0u : a + 1u;
    if (retry_list && !bad)
        for (uint32_t att = 0; att < a; ++att) {        // attempts whose root had failed beforehand
            const uint32_t k = atomicAdd(retry_count, 1u);
            retry_list[2u * k] = s;
            retry_list[2u * k + 1u] = att;
        }
    if (msgs)
        for (uint32_t k = 0; k < nmsg; ++k) msgs[size_t(s) * nmsg + k] = 0ull;
    if (bad)
        for (uint32_t b = 0; b < g.EB; b += 4) *reinterpret_cast<uint32_t*>(result + size_t(s) * g.EB + b) = 0u;
}

// One thread per scenario (or retry entry): the subtrees of the deepest tier that
// are not for the plain register kernel, each once, appended to one of two lists
// (one atomic per wavefront and list: the counters are single hot words): to the
// register kernel with failure handling if that is in use (A.wave_general), else
// to the LDS-tile kernel.
__global__ void __launch_bounds__(256) fixlist_kernel(RunArgs A)
{
    const Geom& g = A.g;
    const uint32_t dlo = A.tiers[0].dlo;
    const uint32_t sv = blockIdx.x * blockDim.x + threadIdx.x;
    const uint32_t F = g.f > 0 ? g.f : 1;
    uint32_t cones[18], nc = 0;
    bool live = sv < A.S + A.retry_slots;
    uint32_t s = sv, root = 0;
    if (live) {
        if (sv < A.S) {
            if (A.status[s] == kStBadFailureSet) live = false;
            else if (A.attempts) root = A.attempts[s] - 1u;
            else if (A.root) root = A.root[s];
        } else {
            const uint32_t kk = sv - A.S;
            if (kk >= *A.retry_count) live = false;
            else { s = A.retry_list[2u * kk]; root = A.retry_list[2u * kk + 1u]; }
        }
    }
    if (live)
        for_each_special_row(g, dlo, A.fail_rank + size_t(s) * F, root, [&](uint32_t jr) {
            const uint32_t c = subtree_of_row(jr, dlo);
            if (c == kNoRank) return;
            bool dup = false;
            for (uint32_t k = 0; k < nc; ++k) dup = dup || cones[k] == c;
            if (!dup) cones[nc++] = c;
        });
    // which list: 0 = LDS tiles, 1 = registers without rows on the deepest level, 2 = registers with such rows
    // (kept apart so that a wavefront of the register kernel walks subtrees of one height)
    const uint32_t top0 = (1u << dlo) - 1u;
    // The register kernels fold all the other subtrees; every process in those sends each of its messages
    // (W - 1 in the up-correction, one in the tree), and the count is a matter of shape: a subtree has all
    // 2^(h+1) - 1 rows (h = kWaveH), or lacks the deepest level; the one in between is on the list.
    if (live && A.msgs) {
        const uint32_t nsub = 1u << dlo;
        uint32_t n_full = ((g.M + 1u) >> kWaveH) - 1u - top0;            // subtrees whose last leaf exists
        uint32_t n_some = (g.M >> kWaveH) - top0;                        // subtrees whose first leaf exists
        n_full = n_full < nsub ? n_full : nsub;
        n_some = n_some < nsub ? n_some : nsub;
        uint32_t n_flat = nsub - n_some;                                 // subtrees without the deepest level
        for (uint32_t k = 0; k < nc; ++k) {
            const uint32_t rs = top0 + cones[k];
            if ((((rs + 2u) << kWaveH) - 2u) < g.M) --n_full;
            else if ((((rs + 1u) << kWaveH) - 1u) >= g.M) --n_flat;
        }
        unsigned long long rows = (unsigned long long)n_full * ((2u << kWaveH) - 1u) +
                                  (unsigned long long)n_flat * ((1u << kWaveH) - 1u);
        if (A.lift) {
            // the levels the plain kernel folds above its subtrees (depths dlo - lift .. dlo - 1, complete rows
            // all): the same count for every row without a listed member; the kernel counts the others
            uint32_t lrows[16], nl = 0;
            for (uint32_t q = 0; q < g.f; ++q) {
                const uint32_t rank = A.fail_rank[size_t(s) * F + q];
                if (rank == kNoRank) continue;
                const uint32_t vr = relabel(rank, root);
                if (vr == 0) continue;                           // the root is in the last row, if in any
                const uint32_t jr = fdiv(vr - 1u, g.divW), d = ilog2(jr + 1u);
                if (d + A.lift < dlo || d >= dlo) continue;
                bool dup = false;
                for (uint32_t k = 0; k < nl; ++k) dup = dup || lrows[k] == jr;
                if (!dup) lrows[nl++] = jr;
            }
            rows += (1u << dlo) - (1u << (dlo - A.lift)) - nl;
        }
        if (rows != 0ull) {
            atomicAdd(&A.msgs[size_t(s) * A.nmsg + 0], rows * g.W * (g.W - 1u));
            atomicAdd(&A.msgs[size_t(s) * A.nmsg + 1], rows * g.W);
        }
    }
    uint32_t kind[18], cnt[3] = {0, 0, 0};
    for (uint32_t k = 0; k < nc; ++k) {
        const bool deep = (((top0 + cones[k] + 1u) << kWaveH) - 1u) < g.M;
        kind[k] = A.wave_general ? (deep ? 2u : 1u) : 0u;
        ++cnt[kind[k]];
    }
    // exclusive prefix sums over the wavefront, one atomic per list
    const uint32_t lane = threadIdx.x & 63u;
    uint32_t at[3];
    for (uint32_t c = 0; c < 3; ++c) {
        uint32_t incl = cnt[c];
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const uint32_t up = __shfl_up(incl, d);
            if (lane >= uint32_t(d)) incl += up;
        }
        const uint32_t total = __shfl(incl, 63);
        uint32_t b = 0;
        if (lane == 0 && total != 0) b = atomicAdd(c == 0 ? A.fix_count : A.wfix_count + (c - 1u), total);
        at[c] = __shfl(b, 0) + incl - cnt[c];
    }
    for (uint32_t k = 0; k < nc; ++k) {            // (scenario or S + retry entry, subtree, scenario, root)
        const vec16_t en = {sv, cones[k], s, root};
        const uint32_t c = kind[k];
        if (c == 0) reinterpret_cast<vec16_t*>(A.fix_list)[at[0]++] = en;
        else if (c == 1) reinterpret_cast<vec16_t*>(A.wfix_list)[at[1]++] = en;
        else reinterpret_cast<vec16_t*>(A.wfix_list)[A.wfix_cap - 1u - at[2]++] = en;
    }
}

// ---------------------------------------------------------------------------
// Which listed processes are DETECTED as failed: a process that is alive waits in vain for a message of the
// failure-free schedule and the failure monitor confirms that the sender has failed (section "Up-Correction",
// last paragraph).  Whether a message of a listed process comes depends on liveness alone (a reduce sends
// whatever it has; in the broadcast a living process that holds no value sends nothing either, but the monitor
// then answers "alive"), so one thread per scenario walks through the messages each listed process has in the
// failure-free schedule of every attempt: to the group mates of the up-correction rounds, to its parent (who
// notices in the round of its own tree message, the root in the last round of the reduce), to its children in
// the broadcast, to the group mates of the correction rounds.

__device__ __forceinline__ bool listed_alive(const Geom& g, const uint32_t* fr, const uint32_t* fo, uint32_t phys,
                                             uint32_t now)
{
    for (uint32_t q = 0; q < g.f; ++q)
        if (fr[q] == phys) return alive_at(fo[q], now);
    return true;
}

__global__ void __launch_bounds__(256) detect_kernel(Geom g, uint32_t kind /* 0 reduce, 1 allreduce */, uint32_t S,
                                                     const uint32_t* root_in, const uint32_t* fail_rank,
                                                     const uint32_t* fail_round, uint32_t* detected)
{
    const uint32_t s = blockIdx.x * blockDim.x + threadIdx.x;
    if (s >= S) return;
    const uint32_t F = g.f > 0 ? g.f : 1;
    const uint32_t* fr = fail_rank + size_t(s) * F;
    const uint32_t* fo = fail_round + size_t(s) * F;
    // the scenario check of the run (prepass_kernel): a bad failure set is not simulated
    bool bad = false;
    uint32_t lead = 0;
    for (uint32_t q = 0; q < F; ++q) {
        const uint32_t r = fr[q];
        if (r == kNoRank) continue;
        if (q >= g.f || r >= g.P) { bad = true; continue; }
        for (uint32_t q2 = 0; q2 < q; ++q2) bad = bad || fr[q2] == r;
        if (kind == 1 && r <= g.f) {
            if (fo[q] != 0) bad = true; else lead |= 1u << r;
        }
    }
    if (kind == 0 && root_in && root_in[s] >= g.P) bad = true;
    uint32_t natt = 1;
    if (kind == 1) while ((lead >> (natt - 1u)) & 1u) ++natt;
    uint32_t mask = 0;
    for (uint32_t att = 0; att < natt && !bad; ++att) {
        const uint32_t root = kind == 1 ? att : (root_in ? root_in[s] : 0u);
        const uint32_t base = kind == 1 ? att * g.Ratt : 0u;
        for (uint32_t q = 0; q < g.f; ++q) {
            if (fr[q] == kNoRank || ((mask >> q) & 1u)) continue;
            const uint32_t fq = fo[q];
            const uint32_t vq = relabel(fr[q], root);
            bool det = false;
            // its place: position j of subtree i (also member i of group j); the root stands in the last group
            uint32_t i = 0, j = 0, gs = 0;
            bool in_group = true;
            if (vq == 0) {
                in_group = g.a > 1;
                j = g.M - 1u; i = g.a - 1u; gs = g.a;
            } else {
                j = fdiv(vq - 1u, g.divW);
                i = vq - 1u - j * g.W;
                gs = group_size(g, j);
            }
            // virtual rank of member r of group j
            auto member = [&](uint32_t r) { return (j == g.M - 1u && g.a > 1 && r == g.a - 1u) ? 0u : 1u + j * g.W + r; };
            for (uint32_t phase = 0; phase < (kind == 1 ? 2u : 1u) && in_group; ++phase) {
                // up-correction rounds 1..f; correction rounds of the broadcast, local rounds Rred + D + 1 ..
                const uint32_t r0 = phase == 0 ? base : base + g.Rred + g.D;
                for (uint32_t t = 1; t <= g.f && t + 1u <= gs && !det; ++t) {
                    const uint32_t now = r0 + t;
                    if (!alive_at(fq, now) && listed_alive(g, fr, fo, relabel(member(exchange_target(i, t, gs)), root), now)) det = true;
                }
            }
            if (vq != 0 && !det) {
                // the tree message, due in the round of its height; the parent looks for it when it sends its own
                const uint32_t sent_round = base + tree_send_round(g, i, j);
                if (!alive_at(fq, sent_round)) {
                    uint32_t pv, pnow;
                    if (j == 0) { pv = 0; pnow = base + g.Rred; }
                    else { const uint32_t jp = sh_parent(g, j); pv = 1u + jp * g.W + i; pnow = base + tree_send_round(g, i, jp); }
                    if (listed_alive(g, fr, fo, relabel(pv, root), pnow)) det = true;
                }
            }
            if (kind == 1 && !det) {
                // broadcast down the tree: its children wait for its message in the round of their depth
                const uint32_t d = vq == 0 ? 0u : sh_depth(g, j);
                const uint32_t now = base + g.Rred + d + 1u;
                if (!alive_at(fq, now)) {
                    if (vq == 0) {
                        for (uint32_t k = 0; k < row_members(g, 0) && !det; ++k)
                            if (listed_alive(g, fr, fo, relabel(1u + k, root), now)) det = true;
                    } else {
                        sh_for_children(g, subtree_size(g, i), j, [&](uint32_t jc) {
                            if (!det && listed_alive(g, fr, fo, relabel(1u + jc * g.W + i, root), now)) det = true;
                        });
                    }
                }
            }
            if (det) mask |= 1u << q;
        }
    }
    detected[s] = mask;
}

// ---------------------------------------------------------------------------
// broadcast half of the allreduce, for the attempt whose root is alive:
// rounds 1..D send the value down the tree (a process at depth d receives in
// round d and forwards in round d+1), rounds D+1..D+f are correction rounds in
// the up-correction groups (every holder sends to group mate (i+t) mod g).
// A workgroup owns `chunk` consecutive physical ranks of one scenario: it works
// out who holds the value (one thread per group), then streams the receive
// buffers.

struct BcastArgs {
    Geom g;
    uint32_t S;
    const uint32_t* attempts;
    const uint32_t* status;
    const uint32_t* fail_rank;
    const uint32_t* fail_round;
    const unsigned char* result;
    uint32_t* has_bitmap;          // or nullptr
    unsigned char* out;            // or nullptr
    unsigned long long* msgs;      // or nullptr
    uint32_t chunk, nchunks;
    FastDiv div_nchunks;
    uint32_t vec16;
    uint32_t small16;              // one value of 4 or 8 bytes per process: several receive buffers per store
    uint32_t any16;                // ALT only: values that are no multiple of 16 bytes, 16 bytes per store
};

struct BcastFail {
    uint32_t listed, cnt_tree, cnt_corr;
    uint32_t touched;          // a listed process stands in a row of this chunk, or above one and did not forward
    uint32_t row[16], idx[16];
    uint32_t recv_alive[16];   // alive in the round in which the value reaches it down the tree
    uint32_t blocked[16];      // dead in the round in which it would forward the value
    uint32_t corr[16];         // number of correction rounds in which it is still alive
};

inline uint32_t bcast_lds_bytes(const BcastArgs& B)
{
    // the failure table, the holder bits of the chunk, and (16-byte stores of odd-sized values) a copy of the result
    return uint32_t(sizeof(BcastFail)) + (B.chunk / 32u + 2u) * 4u + (B.any16 ? B.g.EB : 0u);
}

// BIN: the default tree shape (binary heap inside a subtree), with its index arithmetic known at compile time.
// ALT: the instantiation for small or odd-sized values (not the benchmark's: kept apart, since a branch more in
// this kernel's prologue costs the headline shape several per cent).  It works out the holders and counts of a
// chunk that no listed process touches from the chunk's place in the tree instead of a thread per group (with
// few bytes per process a chunk has many groups, and the kernel is bound by them, not by its stores), and writes
// values that are no multiple of 16 bytes with 16-byte stores (B.any16).
template <bool BIN, bool ALT>
__global__ void __launch_bounds__(kThreads) bcast_kernel(BcastArgs B)
{
    extern __shared__ __align__(16) unsigned char smem[];
    BcastFail& bf = *reinterpret_cast<BcastFail*>(smem);
    uint32_t* bits = reinterpret_cast<uint32_t*>(smem + sizeof(BcastFail));
    const Geom& g = B.g;
    const uint32_t tid = threadIdx.x;
    // Workgroups are dealt to the eight XCDs in turn (workgroup b runs on XCD b mod 8).  The chunks are numbered
    // so that each XCD writes one contiguous eighth of the receive buffers: streams of stores that interleave
    // chunk by chunk over the XCDs reach 5.8 TB/s on this chip, one contiguous region per XCD 6.4 to 7 TB/s.
    uint32_t bid = blockIdx.x;
    const uint32_t per_xcd = gridDim.x >> 3;
    if (bid < (per_xcd << 3)) bid = (bid & 7u) * per_xcd + (bid >> 3);
    const uint32_t s = fdiv(bid, B.div_nchunks);
    const uint32_t ch = bid - s * B.nchunks;
    const uint32_t c0 = ch * B.chunk;
    const uint32_t c1 = c0 + B.chunk < g.P ? c0 + B.chunk : g.P;
    const uint32_t nw = (c1 - c0 + 31u) / 32u;
    const uint32_t NW = (g.P + 31u) / 32u;
    const bool run = B.status[s] == kStOk;

    uint32_t root = 0, t0 = 0;
    // the rows (up-correction groups) with a tree member among the chunk's ranks: virtual ranks vlo .. c1-1
    const uint32_t vlo = c0 > 1u ? c0 : 1u;
    uint32_t j0 = 0, nrows = 0;
    if (vlo < c1) {
        j0 = fdiv(vlo - 1u, g.divW);
        nrows = fdiv(c1 - 2u, g.divW) - j0 + 1u;
    }
    uint32_t jx = kNoRank;                    // the row of the process numbered `root`, which stands at position 0
    for (uint32_t w = tid; w < nw + 1u; w += kThreads) bits[w] = 0u;
    if constexpr (ALT) {
        if (B.any16) {                        // the result's words, at hand for stores that pick them one by one
            uint32_t* resl = bits + (B.chunk / 32u + 2u);
            const uint32_t* resg = reinterpret_cast<const uint32_t*>(B.result + size_t(s) * g.EB);
            for (uint32_t w = tid; w < g.EB / 4u; w += kThreads) resl[w] = resg[w];
        }
    }
    if (run) {
        root = B.attempts[s] - 1u;
        t0 = root * g.Ratt + g.Rred;          // broadcast round tau is global round t0 + tau
        if (root != 0 && c0 == 0) {
            jx = fdiv(root - 1u, g.divW);
            if (jx >= j0 && jx < j0 + nrows) jx = kNoRank;
        }
        if (tid < 64) {
            const uint32_t F = g.f > 0 ? g.f : 1;
            uint32_t row = kNoRank, idx = 0, ra = 0, bl = 0, corr = 0;
            bool used = false;
            if (tid < g.f) {
                uint32_t rank = B.fail_rank[size_t(s) * F + tid];
                if (rank != kNoRank) {
                    uint32_t vr = relabel(rank, root);
                    if (vr != 0) {                 // the root of this attempt is alive, never listed
                        used = true;
                        uint32_t fr = B.fail_round[size_t(s) * F + tid];
                        row = fdiv(vr - 1, g.divW);
                        idx = vr - 1 - row * g.W;
                        uint32_t d = BIN ? depth_of(row) : sh_depth(g, row);
                        ra = alive_at(fr, t0 + d) ? 1u : 0u;
                        bl = alive_at(fr, t0 + d + 1u) ? 0u : 1u;
                        // alive in correction round t iff t0 + D + t < fr
                        uint32_t lim = t0 + g.D + 1u;
                        corr = fr > lim ? fr - lim : 0u;
                        if (corr > 15u) corr = 15u;
                    }
                }
            }
            if (tid < 16) {
                bf.row[tid] = row; bf.idx[tid] = idx; bf.recv_alive[tid] = ra; bf.blocked[tid] = bl;
                bf.corr[tid] = corr;
            }
            // does this entry touch a row of the chunk?  Its own row, or (if it did not forward the value) a row
            // below its own: the rows below row r on the k-th level down are (r+1) 2^k - 1 .. (r+2) 2^k - 2
            bool hit = false;
            if (used) {
                const uint32_t j1 = j0 + nrows;            // one past the last row
                hit = (nrows != 0 && row >= j0 && row < j1) || row == jx;
                if (bl && !BIN) hit = true;       // rows below a position are ranges in the binary heap only
                if (bl && BIN)
                    for (uint32_t k = 1; !hit; ++k) {
                        const uint32_t lo = ((row + 1u) << k) - 1u, hi = ((row + 2u) << k) - 2u;
                        if (lo >= g.M) break;
                        hit = (nrows != 0 && lo < j1 && hi >= j0) || (jx != kNoRank && lo <= jx && jx <= hi);
                    }
            }
            unsigned long long m = __ballot(used);
            unsigned long long mh = __ballot(hit);
            if (tid == 0) {
                bf.listed = uint32_t(__popcll(m));
                bf.cnt_tree = 0;
                bf.cnt_corr = 0;
                bf.touched = mh != 0ull ? 1u : 0u;
            }
        }
    }
    __syncthreads();

    if (ALT && BIN && run && bf.touched == 0u && root == 0) {
        // ---- nobody listed in these rows or above them: every process of the chunk receives, forwards and takes
        // part in every correction round; holders and message counts follow from the chunk's place in the tree
        for (uint32_t w = tid; w < nw; w += kThreads) {
            const uint32_t left = c1 - c0 - 32u * w;
            bits[w] = left >= 32u ? 0xFFFFFFFFu : (1u << left) - 1u;
        }
        if (tid == 0 && B.msgs) {
            // the rows whose first member lies in the chunk count their messages: ja <= j < jb
            const uint32_t ja = c0 <= 1u ? 0u : fdiv(c0 - 1u + g.W - 1u, g.divW);
            uint32_t jb = fdiv(c1 - 1u + g.W - 1u, g.divW);
            if (jb > g.M) jb = g.M;
            unsigned long long tree = 0, corr = 0;
            if (ja < jb) {
                // tree: a message to every member of the children rows 2 ja + 1 .. 2 jb that exist (the last row
                // of the tree may be short)
                const uint32_t lo = 2u * ja + 1u, hi = 2u * jb;
                if (lo < g.M - 1u) tree += (unsigned long long)g.W * ((hi < g.M - 2u ? hi : g.M - 2u) - lo + 1u);
                if (lo <= g.M - 1u && g.M - 1u <= hi) tree += g.nlast;
                // correction: every member of a group sends in each of min(f, group size - 1) rounds
                const uint32_t with_last = jb == g.M ? 1u : 0u;
                const uint32_t gl = group_size(g, g.M - 1u);
                corr = (unsigned long long)(jb - ja - with_last) * g.W * (g.f < g.W - 1u ? g.f : g.W - 1u) +
                       (unsigned long long)with_last * gl * (g.f < gl - 1u ? g.f : gl - 1u);
            }
            if (c0 == 0) tree += g.W;             // the root sends to its f+1 children
            if (tree) atomicAdd(&B.msgs[size_t(s) * 4u + 2u], tree);
            if (corr) atomicAdd(&B.msgs[size_t(s) * 4u + 3u], corr);
        }
    } else if (run) {
        // ---- who holds the value: one thread per up-correction group
        const bool touched = bf.touched != 0u;         // else every process of these rows receives and forwards
        const uint32_t ntask = nrows + (jx != kNoRank ? 1u : 0u);
        uint32_t my_tree = 0, my_corr = 0;
        for (uint32_t t = tid; t < ntask; t += kThreads) {
            const uint32_t j = t < nrows ? j0 + t : jx;
            const uint32_t v0 = 1u + j * g.W;                    // first virtual rank of the row
            const bool owner = t < nrows && v0 >= c0 && v0 < c1; // counts the row's messages
            const uint32_t gs = group_size(g, j);
            const uint32_t nk = row_members(g, j);
            const uint32_t full = (1u << gs) - 1u;
            const uint32_t tmask = (1u << nk) - 1u;
            uint32_t H = tmask;                    // reached down the tree
            if (gs > nk) H |= 1u << (gs - 1u);     // the root, member a-1 of the last group, holds it
            uint32_t blockedm = 0;
            bool rowfail = false;
            if (touched) {
                for (uint32_t q = 0; q < g.f; ++q) {
                    const uint32_t rq = bf.row[q];
                    if (rq == kNoRank) continue;
                    if (rq == j) {
                        rowfail = true;
                        if (!bf.recv_alive[q]) H &= ~(1u << bf.idx[q]);
                        if (bf.blocked[q]) blockedm |= 1u << bf.idx[q];
                    } else if (bf.blocked[q] && bf.idx[q] < nk && (BIN ? is_proper_ancestor(rq, j) : sh_is_proper_ancestor(g, rq, j))) {
                        H &= ~(1u << bf.idx[q]);   // an ancestor in the same subtree did not forward
                    }
                }
            }
            if (owner) {
                // tree-down messages: a holder alive in its send round sends to each child
                const uint32_t snd = H & tmask & ~blockedm;
                if constexpr (BIN) {
                    const uint32_t jc = 2u * j + 1u;
                    const uint32_t m0 = jc < g.M - 1u ? 0xFFFFu : (jc == g.M - 1u ? (1u << g.nlast) - 1u : 0u);
                    const uint32_t m1 = jc + 1u < g.M - 1u ? 0xFFFFu : (jc + 1u == g.M - 1u ? (1u << g.nlast) - 1u : 0u);
                    my_tree += uint32_t(__popc(snd & m0)) + uint32_t(__popc(snd & m1));
                } else {
                    // every child row: all members exist but in the last row, which may be short
                    sh_for_children(g, g.M, j, [&](uint32_t jc) {
                        const uint32_t mc = jc == g.M - 1u ? (1u << g.nlast) - 1u : 0xFFFFu;
                        my_tree += uint32_t(__popc(snd & mc));
                    });
                }
            }
            // correction rounds; where everybody holds the value and lives, each of them sends in every round
            if (!rowfail && H == full) {
                if (owner) my_corr += gs * (g.f < gs - 1u ? g.f : gs - 1u);
            } else {
                for (uint32_t tt = 1; tt <= g.f && tt + 1u <= gs; ++tt) {
                    uint32_t am = full;
                    if (rowfail)
                        for (uint32_t q = 0; q < g.f; ++q)
                            if (bf.row[q] == j && bf.corr[q] < tt) am &= ~(1u << bf.idx[q]);
                    const uint32_t snd = H & am;
                    if (owner) my_corr += uint32_t(__popc(snd));
                    H |= exchange_targets(snd, tt, gs, full) & am;
                }
            }
            // record the holders among the row's tree members, by physical rank
            uint32_t Hm = H & tmask;
            if (root != 0 && root >= v0 && root < v0 + nk) {
                const uint32_t b = root - v0;
                if (((Hm >> b) & 1u) && c0 == 0) atomicOr(&bits[0], 1u);
                Hm &= ~(1u << b);
            }
            if (t < nrows) {
                int rel = int(v0) - int(c0);
                if (rel < 0) { Hm >>= uint32_t(-rel); rel = 0; }
                const uint32_t room = c1 - c0 - uint32_t(rel);        // ranks of the chunk from rel on
                if (room < 32u) Hm &= (1u << room) - 1u;
                const unsigned long long wide = (unsigned long long)Hm << (uint32_t(rel) & 31u);
                const uint32_t w0 = uint32_t(rel) >> 5;
                if (uint32_t(wide)) atomicOr(&bits[w0], uint32_t(wide));
                if (uint32_t(wide >> 32)) atomicOr(&bits[w0 + 1u], uint32_t(wide >> 32));
            }
        }
        if (tid == 0) {
            if (root >= c0 && root < c1) atomicOr(&bits[(root - c0) >> 5], 1u << ((root - c0) & 31u));
            if (c0 == 0) my_tree += g.W;          // the root sends to its f+1 children
        }
        if (B.msgs) {
            if (my_tree) atomicAdd(&bf.cnt_tree, my_tree);
            if (my_corr) atomicAdd(&bf.cnt_corr, my_corr);
        }
    }
    __syncthreads();

    if (run && B.msgs && tid == 0) {
        if (bf.cnt_tree) atomicAdd(&B.msgs[size_t(s) * 4u + 2u], (unsigned long long)bf.cnt_tree);
        if (bf.cnt_corr) atomicAdd(&B.msgs[size_t(s) * 4u + 3u], (unsigned long long)bf.cnt_corr);
    }
    if (B.has_bitmap)
        for (uint32_t w = tid; w < nw; w += kThreads) B.has_bitmap[size_t(s) * NW + (c0 >> 5) + w] = bits[w];

    // ---- receive buffers: the value where held, zeros elsewhere
    if (B.out) {
        unsigned char* dst = B.out + (size_t(s) * g.P + c0) * g.EB;
        const unsigned char* res = B.result + size_t(s) * g.EB;
        const uint32_t bytes = (c1 - c0) * g.EB;
        if (B.vec16 && (kThreads * 16u) % g.EB == 0u) {
            // a thread's 16 bytes sit at the same place of a value in every pass: one load of the result
            const uint32_t o0 = tid * 16u;
            const uint32_t r0 = fdiv(o0, g.divEB);
            const vec16_t mine = *reinterpret_cast<const vec16_t*>(res + (o0 - r0 * g.EB));
            const vec16_t zero = {0u, 0u, 0u, 0u};
            const uint32_t rstep = (kThreads * 16u) / g.EB;
            uint32_t rr = r0;
            for (uint32_t o = o0; o < bytes; o += kThreads * 16u, rr += rstep) {
                const bool has = ((bits[rr >> 5] >> (rr & 31u)) & 1u) != 0u;
                __builtin_nontemporal_store(has ? mine : zero, reinterpret_cast<vec16_t*>(dst + o));   // written once, read by others
            }
        } else if (B.small16) {
            // 16 bytes = the receive buffers of 16 / EB consecutive processes
            const uint32_t per = 16u / g.EB, wpr = g.EB / 4u;         // processes per store, words per value
            const uint32_t r0w = reinterpret_cast<const uint32_t*>(res)[0];
            const uint32_t r1w = wpr > 1u ? reinterpret_cast<const uint32_t*>(res)[1] : r0w;
            const uint32_t nvec = bytes / 16u;                       // whole: P * EB is a multiple of 16, so is the chunk
            for (uint32_t i = tid; i < nvec; i += kThreads) {
                const uint32_t rr = i * per;
                const uint32_t m = (bits[rr >> 5] >> (rr & 31u));    // per <= 4 and rr % per == 0: same word
                vec16_t val;
                if (wpr == 2u) {
                    val.x = (m & 1u) ? r0w : 0u; val.y = (m & 1u) ? r1w : 0u;
                    val.z = (m & 2u) ? r0w : 0u; val.w = (m & 2u) ? r1w : 0u;
                } else {
                    val.x = (m & 1u) ? r0w : 0u; val.y = (m & 2u) ? r0w : 0u;
                    val.z = (m & 4u) ? r0w : 0u; val.w = (m & 8u) ? r0w : 0u;
                }
                __builtin_nontemporal_store(val, reinterpret_cast<vec16_t*>(dst + size_t(i) * 16u));
            }
        } else if (ALT && B.any16) {
            // 16 bytes = four words, each of some process's receive buffer: the store walks along with (process,
            // word of its value); P * EB is a multiple of 16, so the chunk ends on a store
            const uint32_t* resw = bits + (B.chunk / 32u + 2u);       // the kernel's copy of the result in LDS
            const uint32_t wpv = g.EB / 4u;                          // words per value
            for (uint32_t o = tid * 16u; o < bytes; o += kThreads * 16u) {
                uint32_t rr = fdiv(o, g.divEB);
                uint32_t wi = (o - rr * g.EB) / 4u;
                uint32_t v[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    v[k] = ((bits[rr >> 5] >> (rr & 31u)) & 1u) ? resw[wi] : 0u;
                    if (++wi == wpv) { wi = 0; ++rr; }
                }
                const vec16_t val = {v[0], v[1], v[2], v[3]};
                __builtin_nontemporal_store(val, reinterpret_cast<vec16_t*>(dst + o));
            }
        } else if (B.vec16) {
            for (uint32_t o = tid * 16u; o < bytes; o += kThreads * 16u) {
                const uint32_t rr = fdiv(o, g.divEB);
                const uint32_t within = o - rr * g.EB;
                uint4 val = make_uint4(0, 0, 0, 0);
                if ((bits[rr >> 5] >> (rr & 31u)) & 1u) val = *reinterpret_cast<const uint4*>(res + within);
                *reinterpret_cast<uint4*>(dst + o) = val;
            }
        } else {
            for (uint32_t o = tid * 4u; o < bytes; o += kThreads * 4u) {
                const uint32_t rr = fdiv(o, g.divEB);
                const uint32_t within = o - rr * g.EB;
                uint32_t val = 0;
                if ((bits[rr >> 5] >> (rr & 31u)) & 1u) val = *reinterpret_cast<const uint32_t*>(res + within);
                *reinterpret_cast<uint32_t*>(dst + o) = val;
            }
        }
    }
}

}  // namespace ftred

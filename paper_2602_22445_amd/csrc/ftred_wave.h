// Deepest tier of the tree phase: one LANE walks one subtree of rows, in registers.
//
// A row (= one up-correction group = the j-th process of each subtree of the
// root) is W*E values that are consecutive in HBM: [member k][value index e].
// A lane owns (subtree, value index e): it visits the 31 rows of its subtree of
// height 4 in post-order, loads the W inputs of each row (one load per member),
// forms the W up-correction values in the order of the rounds (Algorithm
// "Up-correction"), adds the tree messages of the two children rows, which are its
// own earlier results (Algorithm "reduce at non-roots"), and ends with the W tree
// messages of the subtree's top row.  Nothing is exchanged between lanes: no LDS,
// no barrier, no shuffle.  The 64 lanes of a wavefront are ne value indices times
// 64/ne sibling subtrees; the lanes of one subtree read consecutive values, and the
// W loads of a row use every byte of it.  A ring of rows per lane is requested
// ahead of the fold.
//
// This kernel runs the subtrees in which every row exists (with or without the
// bottom level), nobody is listed as failed and the short last group does not
// occur; a root other than process 0 is handled here (the relabelled rank's input
// is swapped in).  The few others (at most f + 1 per scenario) are listed by a
// small kernel of their own and run by the list kernels (ftred_wave_general.h, or
// the LDS-tile kernel when the lists of failed processes are asked for), which
// carry per-member liveness, sent and failed bits (section "Failure information":
// the single failed bit); here they are skipped.  A wavefront walks through one or
// more groups of sibling subtrees; its groups lie a stride of wavefronts apart.
//
// The subtree's top row leaves through the scratch area in the format the upper
// tiers read: W*E values and one word (bits 0..15 sent, 16..31 failed bit).
// The messages of these subtrees (every process in them sends all of its own) are
// counted by the kernel that lists the other subtrees: their number follows from
// the shape of the tree and that list.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ftred_geom.h"
#include "ftred_kernels.h"

namespace ftred {

constexpr int kWaveH = 4;            // height of the subtree one lane walks
constexpr int kWaveThreads = 64;     // one wavefront per workgroup: lanes are independent
constexpr uint32_t kWaveRows = (2u << kWaveH) - 1u;

struct WaveLayout {                  // how the 64 lanes map to (subtree slot, value index)
    uint32_t ne;                     // value indices per pass
    uint32_t slot_shift;             // 2^slot_shift sibling subtrees per wavefront
    uint32_t nact;                   // active lanes = slots * ne
    uint32_t passes;                 // ceil(E / ne)
    uint32_t group_shift;            // a wavefront walks through 2^group_shift groups of subtrees
    uint32_t stage;                  // 1: the top rows of all its groups wait in LDS for one run of stores at the end
};

// LDS of one wavefront when the top rows are staged: the rows, then one word per subtree
inline uint32_t wave_lds_bytes(const Geom& g, const WaveLayout& w)
{
    const uint32_t cones = 1u << (w.group_shift + w.slot_shift);
    return w.stage ? cones * g.RB + cones * 4u : 0u;
}

// staging needs all value indices in one pass and a modest tile
inline bool wave_can_stage(const Geom& g, const WaveLayout& w)
{
    return w.passes == 1u && g.RB % 8u == 0u && (uint64_t(g.RB + 4u) << (w.group_shift + w.slot_shift)) <= 12u * 1024u;
}

// Group widths the register kernels are built for (straight-line code per width).  The plain walks (one lane per
// subtree, eight lanes per subtree) exist for W = f + 1 = 2 .. 16; a lane holds (rows in flight + levels + 1) * W
// values, which is two wavefronts per SIMD at W = 10, 11 and one from W = 12 on (still several times faster than LDS
// tiles).  The walk with failure handling and the kernel that folds a whole scenario are built for W <= 9 only:
// W * (W - 1) predicated additions per visit, 31 visits, take minutes to compile per width, value type and
// operator (all widths: a build of 16 instead of 4 minutes); for wider groups the listed subtrees run on the
// LDS-tile list kernel.
constexpr uint32_t kWaveMinW = 2, kWaveMaxW = 16, kWaveListMaxW = 9;
inline bool wave_width_ok(uint32_t W) { return W >= kWaveMinW && W <= kWaveMaxW; }
inline bool wave_list_width_ok(uint32_t W) { return W >= kWaveMinW && W <= kWaveListMaxW; }

// `return FN<W>(args...)` for the run-time group width W: the widths of the walk with failure handling and the
// fused kernel, and all widths of the plain walks
#define FTRED_WAVE_WIDTH_SWITCH(W, FN, ...)                     \
    switch (W) {                                                \
        case 2: return FN<2>(__VA_ARGS__);                      \
        case 3: return FN<3>(__VA_ARGS__);                      \
        case 4: return FN<4>(__VA_ARGS__);                      \
        case 5: return FN<5>(__VA_ARGS__);                      \
        case 6: return FN<6>(__VA_ARGS__);                      \
        case 7: return FN<7>(__VA_ARGS__);                      \
        case 8: return FN<8>(__VA_ARGS__);                      \
        case 9: return FN<9>(__VA_ARGS__);                      \
        default: return hipErrorInvalidValue;                   \
    }
#define FTRED_WAVE_WIDTH_SWITCH_WIDE(W, FN, ...)                \
    switch (W) {                                                \
        case 2: return FN<2>(__VA_ARGS__);                      \
        case 3: return FN<3>(__VA_ARGS__);                      \
        case 4: return FN<4>(__VA_ARGS__);                      \
        case 5: return FN<5>(__VA_ARGS__);                      \
        case 6: return FN<6>(__VA_ARGS__);                      \
        case 7: return FN<7>(__VA_ARGS__);                      \
        case 8: return FN<8>(__VA_ARGS__);                      \
        case 9: return FN<9>(__VA_ARGS__);                      \
        case 10: return FN<10>(__VA_ARGS__);                    \
        case 11: return FN<11>(__VA_ARGS__);                    \
        case 12: return FN<12>(__VA_ARGS__);                    \
        case 13: return FN<13>(__VA_ARGS__);                    \
        case 14: return FN<14>(__VA_ARGS__);                    \
        case 15: return FN<15>(__VA_ARGS__);                    \
        case 16: return FN<16>(__VA_ARGS__);                    \
        default: return hipErrorInvalidValue;                   \
    }

inline WaveLayout make_wave_layout(const Geom& g, uint32_t dlo)
{
    WaveLayout w;
    w.ne = g.E < 64u ? g.E : 64u;
    uint32_t slots = 64u / w.ne, sh = 0;
    while ((2u << sh) <= slots && sh < dlo) ++sh;
    w.slot_shift = sh;
    w.nact = (1u << sh) * w.ne;
    w.passes = (g.E + w.ne - 1u) / w.ne;
    // Four groups per wavefront with the top rows staged in LDS where a scenario still has four wavefronts or more
    // then (P = 16384, f = 4, 8 values: 0.88 ms against 0.91 ms with one group); else one group (P = 1024, f = 3,
    // 16 values: 1.80 ms against 1.83 ms with two or four).  The plan's flags can ask for another number.
    w.group_shift = 0;
    w.stage = 0;
    if (dlo >= sh + 4u) {
        w.group_shift = 2;
        if (wave_can_stage(g, w)) w.stage = 1;
        else w.group_shift = 0;
    }
    return w;
}

constexpr int cx_ilog2(int x) { return x <= 1 ? 0 : 1 + cx_ilog2(x / 2); }

// heap index (top 0, children 2i+1 and 2i+2) of the n-th row in post-order of a
// complete binary tree of height H
constexpr int cx_postorder(int n, int H, int top = 0)
{
    if (H == 0) return top;
    const int sub = (1 << H) - 1;                   // rows below one child
    if (n < sub) return cx_postorder(n, H - 1, 2 * top + 1);
    if (n < 2 * sub) return cx_postorder(n - sub, H - 1, 2 * top + 2);
    return top;
}

// rows requested ahead of the fold: what the registers allow
template <int WP>
struct WaveDepth { static constexpr int value = WP <= 5 ? 4 : 2; };

// One lane's walk through its subtree of height HH below row rs.  bk[k] = the
// scenario's payload + k*EB (wave-uniform), ecol = the lane's value index.
// bottom == false: the lane's subtree lacks its deepest level (the rows of level
// HH - 1 are leaves; only with HH == kWaveH, where lanes of one wavefront may
// differ).  Leaves the W tree messages of row rs in cur.  W == WP.  The visits are
// numbered at compile time (template recursion), so every array index is a constant
// and the arrays live in registers.
// SWAP: the root is not process 0, so the process that carries the root's number
// (virtual rank `root`, member kx of row jx) is process 0 (section "Reduce": the
// root swaps numbers with process 0): its input x0 replaces what the row's place in
// memory holds, which is the root's own input.
template <class T, int OP, int WP, int HH, bool SWAP>
struct SubtreeWalk {
    static constexpr int PD = WaveDepth<WP>::value;
    static constexpr int NR = (2 << HH) - 1;
    const Geom& g;
    const unsigned char* const (&bk)[WP];
    uint32_t rs, ecol;
    bool bottom;
    uint32_t jx, kx;               // SWAP only
    T x0;
    T xq[PD][WP];                  // rows in flight
    T st[HH + 1][WP];              // finished lower-numbered children waiting for their sibling, by level
    T cur[WP];                     // the row finished last: a higher-numbered child, or the top

    __device__ __forceinline__ SubtreeWalk(const Geom& g_, const unsigned char* const (&bk_)[WP], uint32_t rs_,
                                           uint32_t ecol_, bool bottom_)
        : g(g_), bk(bk_), rs(rs_), ecol(ecol_), bottom(bottom_) {}

    template <int N>
    __device__ __forceinline__ void issue()
    {
        constexpr int li = cx_postorder(N, HH);
        constexpr int l = cx_ilog2(li + 1);
        const uint32_t j = ((rs + 1u) << l) - 1u + uint32_t(li - ((1 << l) - 1));       // the lane's row
        uint32_t off = ((1u + j * g.W) * g.E + ecol) * g.esz;
        if (l == HH) off = bottom ? off : ecol * g.esz;         // a row that does not exist: any valid address
#pragma unroll
        for (int k = 0; k < WP; ++k) xq[N % PD][k] = *reinterpret_cast<const T*>(bk[k] + off);
    }

    template <int N>
    __device__ __forceinline__ void visit()
    {
        constexpr int li = cx_postorder(N, HH);
        constexpr int l = cx_ilog2(li + 1);
        // the row is consumed here and not earlier: without this the compiler moves the
        // additions up to the loads and waits for each row as soon as it is requested
#pragma unroll
        for (int k = 0; k < WP; ++k) asm volatile("" : "+v"(xq[N % PD][k]) : : "memory");
        if constexpr (SWAP) {
            const uint32_t j = ((rs + 1u) << l) - 1u + uint32_t(li - ((1 << l) - 1));
            const bool here = j == jx;
#pragma unroll
            for (int k = 0; k < WP; ++k) xq[N % PD][k] = (here && kx == uint32_t(k)) ? x0 : xq[N % PD][k];
        }
        // up-correction: in round t member i receives the input of member (i - t) mod W
        T v[WP];
#pragma unroll
        for (int i = 0; i < WP; ++i) {
            T acc = xq[N % PD][i];
#pragma unroll
            for (int t = 1; t < WP; ++t) acc = comb<T, OP>(acc, xq[N % PD][exchange_source(uint32_t(i), uint32_t(t), uint32_t(WP))]);
            v[i] = acc;
        }
        if constexpr (N + PD < NR) issue<N + PD>();            // the ring slot is free again
        // tree phase: the lower-numbered child's message first
        if constexpr (l < HH) {
#pragma unroll
            for (int k = 0; k < WP; ++k) {
                const T sum = comb<T, OP>(comb<T, OP>(v[k], st[l + 1][k]), cur[k]);
                v[k] = (l < HH - 1 || bottom) ? sum : v[k];
            }
        }
        if constexpr (li != 0 && (li & 1)) {
#pragma unroll
            for (int k = 0; k < WP; ++k) st[l][k] = v[k];
        } else {
#pragma unroll
            for (int k = 0; k < WP; ++k) cur[k] = v[k];
        }
        if constexpr (N + 1 < NR) visit<N + 1>();
    }

    template <int N>
    __device__ __forceinline__ void prime()
    {
        if constexpr (N < PD && N < NR) {
            issue<N>();
            prime<N + 1>();
        }
    }

    __device__ __forceinline__ void run()
    {
        prime<0>();
        visit<0>();
    }

    // the same with the relabelled rank: root = the root's number (not 0), pay = the scenario's payload
    __device__ __forceinline__ void run_swapped(uint32_t root, const unsigned char* pay)
    {
        jx = fdiv(root - 1u, g.divW);
        kx = root - 1u - jx * g.W;
        x0 = *reinterpret_cast<const T*>(pay + size_t(ecol) * g.esz);
        prime<0>();
        visit<0>();
    }
};

// The subtree (of height kWaveH below a row of depth dlo) that holds row jr: its
// number among the subtrees of that depth, or kNoRank if the row lies above or
// below them.
__device__ __forceinline__ uint32_t subtree_of_row(uint32_t jr, uint32_t dlo)
{
    if (jr == kNoRank) return kNoRank;
    const uint32_t d = ilog2(jr + 1u);
    if (d < dlo || d > dlo + uint32_t(kWaveH)) return kNoRank;
    return ((jr + 1u) >> (d - dlo)) - (1u << dlo);
}

// Rows that take a subtree out of the register kernel, for one (scenario, root):
// the rows of the listed processes, and the last row when the root is a member of
// its group or the bottom level of its subtree is incomplete.  At most f + 1 rows;
// fn(row) is called for each.  Used by the kernel that lists those subtrees and by the register kernel
// that skips them: both must agree.
template <class Fn>
__device__ __forceinline__ void for_each_special_row(const Geom& g, uint32_t dlo, const uint32_t* fail_rank_s,
                                                     uint32_t root, Fn fn)
{
    for (uint32_t q = 0; q < g.f; ++q) {
        const uint32_t rank = fail_rank_s[q];
        if (rank == kNoRank) continue;
        const uint32_t vr = relabel(rank, root);
        const uint32_t jr = vr == 0 ? (g.a > 1 ? g.M - 1u : kNoRank) : fdiv(vr - 1u, g.divW);
        if (jr != kNoRank) fn(jr);
    }
    // the last row: short group with the root in it, or a subtree whose deepest level stops early
    const uint32_t c = subtree_of_row(g.M - 1u, dlo);
    if (c != kNoRank) {
        const uint32_t rs = (1u << dlo) - 1u + c;
        const uint32_t first_leaf = ((rs + 1u) << kWaveH) - 1u, last_leaf = ((rs + 2u) << kWaveH) - 2u;
        const bool ragged = first_leaf < g.M && last_leaf >= g.M;
        if (g.a > 1 || ragged) fn(g.M - 1u);
    }
}

// The same rows, one per lane of a wavefront (f + 1 <= 64): lane e < f takes entry e of the
// failure list (`rank` = that entry, read by the caller), lane f the last row.  Returns the
// lane's row or kNoRank.
__device__ __forceinline__ uint32_t special_row_of_lane(const Geom& g, uint32_t dlo, uint32_t rank, uint32_t root,
                                                        uint32_t lane)
{
    if (lane < g.f) {
        if (rank == kNoRank) return kNoRank;
        const uint32_t vr = relabel(rank, root);
        return vr == 0 ? (g.a > 1 ? g.M - 1u : kNoRank) : fdiv(vr - 1u, g.divW);
    }
    if (lane == g.f) {
        const uint32_t c = subtree_of_row(g.M - 1u, dlo);
        if (c != kNoRank) {
            const uint32_t rs = (1u << dlo) - 1u + c;
            const uint32_t first_leaf = ((rs + 1u) << kWaveH) - 1u, last_leaf = ((rs + 2u) << kWaveH) - 2u;
            const bool ragged = first_leaf < g.M && last_leaf >= g.M;
            if (g.a > 1 || ragged) return g.M - 1u;
        }
    }
    return kNoRank;
}

template <class T, int OP, int WP>
__global__ void __launch_bounds__(kWaveThreads) wave_tier_kernel(RunArgs A, WaveLayout wl)
{
    const Geom& g = A.g;
    const TierDesc& td = A.tiers[0];
    const uint32_t lane = threadIdx.x;
    // a wavefront walks through 2^group_shift consecutive groups of 2^slot_shift sibling subtrees of one scenario
    const uint32_t wshift = td.dlo - wl.slot_shift - wl.group_shift;   // wavefronts per scenario = 2^wshift
    const uint32_t sv = blockIdx.x >> wshift;                  // scenario, or S + retry entry
    const uint32_t top0 = (1u << td.dlo) - 1u;
    // the groups of a wavefront lie 2^wshift groups apart: wavefronts that run side by side read rows that lie side
    // by side whichever of its groups each of them has reached
    const uint32_t wid = blockIdx.x & ((1u << wshift) - 1u);
    if (top0 + (wid << wl.slot_shift) >= g.M) return;          // no such rows
    // staged top rows: [group][slot][member][value index], then one word per (group, slot): folded here
    extern __shared__ __align__(16) unsigned char wave_lds[];
    const uint32_t ncones = 1u << (wl.group_shift + wl.slot_shift);
    T* tile = reinterpret_cast<T*>(wave_lds);
    uint32_t* folded = reinterpret_cast<uint32_t*>(wave_lds + size_t(ncones) * g.RB);
    if (wl.stage) {
        for (uint32_t c = threadIdx.x; c < ncones; c += kWaveThreads) folded[c] = 0u;
        __syncthreads();
    }

    // lane -> (subtree slot, value index e)
    const uint32_t slot = lane / wl.ne;
    const uint32_t e = lane - slot * wl.ne;
    const bool active = lane < wl.nact;

    uint32_t s = sv, root = 0, status = kStOk;
    unsigned char* wsS;
    const uint32_t F = g.f > 0 ? g.f : 1;
    if (sv < A.S) {
        status = A.status[s];
        if (A.attempts) root = A.attempts[s];                  // roots tried; the last one is alive
        else if (A.root) root = A.root[s];
        if (A.attempts) root = root > 0 ? root - 1u : 0u;
        wsS = A.ws + size_t(s) * A.ws_stride;
    } else {
        const uint32_t kk = sv - A.S;
        if (kk >= *A.retry_count) return;
        s = __builtin_amdgcn_readfirstlane(A.retry_list[2u * kk]);
        root = A.retry_list[2u * kk + 1u];
        wsS = A.retry_ws + size_t(kk) * A.ws_stride;
    }
    status = __builtin_amdgcn_readfirstlane(status);
    root = __builtin_amdgcn_readfirstlane(root);
    if (status == kStBadFailureSet) return;
    // the subtrees that go to the list kernels, one per lane (at most f + 1 of them): worked out once and side by
    // side; a loop over the failure list in every lane, in front of every group, delayed the first rows of the walk
    const uint32_t listed = lane < g.f ? A.fail_rank[size_t(s) * F + lane] : kNoRank;
    const uint32_t special = subtree_of_row(special_row_of_lane(g, td.dlo, listed, root, lane), td.dlo);
    const unsigned char* pay = A.payload + size_t(s) * A.scen_stride_bytes;
    const unsigned char* bk[WP];
#pragma unroll
    for (int k = 0; k < WP; ++k) bk[k] = pay + size_t(k) * g.EB;

    for (uint32_t gi = 0; gi < (1u << wl.group_shift); ++gi) {
        const uint32_t cone_w = (wid + (gi << wshift)) << wl.slot_shift;
        if (top0 + cone_w >= g.M) break;                       // no such rows
        const uint32_t cone = cone_w + (active ? slot : 0u);
        const uint32_t rs = top0 + cone;                       // top row of the lane's subtree
        const bool exists = active && rs < g.M;

        // shape of the lane's subtree: complete with or without the bottom level (a ragged one is listed)
        const uint32_t last_leaf = ((rs + 2u) << kWaveH) - 2u;
        const bool bottom = last_leaf < g.M;
        // subtrees on the list of the general (LDS tile) kernel are not for this one
        bool handover = false;
        unsigned long long hits = __ballot(special - cone_w < (1u << wl.slot_shift));    // rarely any
        while (hits != 0ull) {
            const int en = __ffsll(hits) - 1;
            hits &= hits - 1ull;
            if (uint32_t(__builtin_amdgcn_readlane(int(special), en)) == cone) handover = true;
        }
        const bool mine = exists && !handover;
        const bool any_bottom = __ballot(mine && bottom) != 0ull;  // else no lane here has the deepest level

        for (uint32_t pass = 0; pass < wl.passes; ++pass) {
            const uint32_t ecol = pass * wl.ne + e;
            if (mine && ecol < g.E) {
                T out[WP];
                if (root == 0) {
                    if (any_bottom) {
                        SubtreeWalk<T, OP, WP, kWaveH, false> w(g, bk, rs, ecol, bottom);
                        w.run();
#pragma unroll
                        for (int k = 0; k < WP; ++k) out[k] = w.cur[k];
                    } else {
                        SubtreeWalk<T, OP, WP, kWaveH - 1, false> w(g, bk, rs, ecol, true);
                        w.run();
#pragma unroll
                        for (int k = 0; k < WP; ++k) out[k] = w.cur[k];
                    }
                } else {
                    if (any_bottom) {
                        SubtreeWalk<T, OP, WP, kWaveH, true> w(g, bk, rs, ecol, bottom);
                        w.run_swapped(root, pay);
#pragma unroll
                        for (int k = 0; k < WP; ++k) out[k] = w.cur[k];
                    } else {
                        SubtreeWalk<T, OP, WP, kWaveH - 1, true> w(g, bk, rs, ecol, true);
                        w.run_swapped(root, pay);
#pragma unroll
                        for (int k = 0; k < WP; ++k) out[k] = w.cur[k];
                    }
                }
                if (wl.stage) {
                    // the top row waits in LDS: a run of stores per group would hold up the rows requested after it
                    const uint32_t at = (gi << wl.slot_shift) + slot;
#pragma unroll
                    for (int k = 0; k < WP; ++k) tile[(size_t(at) * WP + k) * g.E + ecol] = out[k];
                    if (ecol == 0) folded[at] = 1u;
                    continue;
                }
                // the top row of the subtree goes to the tier above
                unsigned char* dst = wsS + td.out_off + size_t(cone) * g.RB + size_t(ecol) * g.esz;
#pragma unroll
                for (int k = 0; k < WP; ++k) *reinterpret_cast<T*>(dst + size_t(k) * g.EB) = out[k];
                if (ecol == 0) {
                    reinterpret_cast<uint32_t*>(wsS + td.out_meta_off)[cone] = (1u << g.W) - 1u;   // all sent, no failed bit
                    if (A.info) {         // and nobody in the subtree missed a message: empty lists
                        uint16_t* mk = reinterpret_cast<uint16_t*>(wsS + td.out_mask_off) + size_t(cone) * g.W;
#pragma unroll
                        for (int k = 0; k < WP; ++k) mk[k] = 0;
                    }
                }
            }
        }
    }
    if (wl.stage) {
        __syncthreads();
        const uint32_t RE = g.W * g.E, smask = (1u << wl.slot_shift) - 1u;
        auto cone_of = [&](uint32_t c) { return ((wid + ((c >> wl.slot_shift) << wshift)) << wl.slot_shift) + (c & smask); };
        T* dst = reinterpret_cast<T*>(wsS + td.out_off);
        for (uint32_t i = lane; i < ncones * RE; i += kWaveThreads) {
            const uint32_t c = fdiv(i * g.esz, g.divRB);
            if (folded[c]) dst[size_t(cone_of(c)) * RE + (i - c * RE)] = tile[i];
        }
        for (uint32_t c = lane; c < ncones; c += kWaveThreads)
            if (folded[c]) reinterpret_cast<uint32_t*>(wsS + td.out_meta_off)[cone_of(c)] = (1u << g.W) - 1u;
        if (A.info) {
            uint16_t* mk = reinterpret_cast<uint16_t*>(wsS + td.out_mask_off);
            for (uint32_t i = lane; i < ncones * g.W; i += kWaveThreads) {
                const uint32_t c = fdiv(i, g.divW);
                if (folded[c]) mk[size_t(cone_of(c)) * g.W + (i - c * g.W)] = 0;
            }
        }
    }
}

#define FTRED_DECLARE_WAVE_LAUNCHER(NAME) \
    hipError_t launch_wave_##NAME(const RunArgs& A, const WaveLayout& wl, uint32_t grid, hipStream_t st);

FTRED_DECLARE_WAVE_LAUNCHER(i64_sum)
FTRED_DECLARE_WAVE_LAUNCHER(i64_bor)
FTRED_DECLARE_WAVE_LAUNCHER(u32_sum)
FTRED_DECLARE_WAVE_LAUNCHER(u32_bor)
FTRED_DECLARE_WAVE_LAUNCHER(f64_sum)

#define FTRED_DEFINE_WAVE_LAUNCHER(NAME, T, OP)                                                     \
    template <int WP>                                                                               \
    static hipError_t wave_wp_##NAME(const RunArgs& A, const WaveLayout& wl, uint32_t grid, hipStream_t st) \
    {                                                                                               \
        hipLaunchKernelGGL((wave_tier_kernel<T, OP, WP>), dim3(grid), dim3(kWaveThreads),           \
                           wave_lds_bytes(A.g, wl), st, A, wl);                                     \
        return hipGetLastError();                                                                   \
    }                                                                                               \
    hipError_t launch_wave_##NAME(const RunArgs& A, const WaveLayout& wl, uint32_t grid, hipStream_t st) \
    {                                                                                               \
        FTRED_WAVE_WIDTH_SWITCH_WIDE(A.g.W, wave_wp_##NAME, A, wl, grid, st)                        \
    }

}  // namespace ftred

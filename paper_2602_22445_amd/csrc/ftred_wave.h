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
// bottom level), nothing is listed as failed, and neither the relabelled ranks nor
// the short last group occur.  The few others (at most f + 3 per scenario) are
// appended to a list and run by the general LDS-tile kernel, which carries
// per-member liveness, sent and failed bits (section "Failure information": the
// single failed bit).
//
// The subtree's top row leaves through the scratch area in the format the upper
// tiers read: W*E values and one word (bits 0..15 sent, 16..31 failed bit).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ftred_geom.h"
#include "ftred_kernels.h"

namespace ftred {

constexpr int kWaveH = 4;            // height of the subtree one lane walks
constexpr int kWaveThreads = 64;     // one wavefront per workgroup: lanes are independent

struct WaveLayout {                  // how the 64 lanes map to (subtree slot, value index)
    uint32_t ne;                     // value indices per pass
    uint32_t slot_shift;             // 2^slot_shift sibling subtrees per wavefront
    uint32_t nact;                   // active lanes = slots * ne
    uint32_t passes;                 // ceil(E / ne)
};

// group widths the kernel is built for (straight-line code per width)
inline bool wave_width_ok(uint32_t W) { return W == 2 || W == 3 || W == 4 || W == 5 || W == 9; }

inline WaveLayout make_wave_layout(const Geom& g, uint32_t dlo)
{
    WaveLayout w;
    w.ne = g.E < 64u ? g.E : 64u;
    uint32_t slots = 64u / w.ne, sh = 0;
    while ((2u << sh) <= slots && sh < dlo) ++sh;
    w.slot_shift = sh;
    w.nact = (1u << sh) * w.ne;
    w.passes = (g.E + w.ne - 1u) / w.ne;
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

template <int WP>
struct WaveDepth { static constexpr int value = WP <= 5 ? 4 : 2; };     // rows requested ahead

// One lane's walk through its subtree of height HH below row rs.  bk[k] = the
// scenario's payload + k*EB (wave-uniform), ecol = the lane's value index.
// bottom == false: the lane's subtree lacks its deepest level (the rows of level
// HH - 1 are leaves; only with HH == kWaveH, where lanes of one wavefront may
// differ).  Leaves the W tree messages of row rs in cur.  W == WP.  The visits are
// numbered at compile time (template recursion), so every array index is a constant
// and the arrays live in registers.
template <class T, int OP, int WP, int HH>
struct SubtreeWalk {
    static constexpr int PD = WaveDepth<WP>::value;
    static constexpr int NR = (2 << HH) - 1;
    const Geom& g;
    const unsigned char* const (&bk)[WP];
    uint32_t rs, ecol;
    bool bottom;
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
        // up-correction: in round t member i receives the input of member (i - t) mod W
        T v[WP];
#pragma unroll
        for (int i = 0; i < WP; ++i) {
            T acc = xq[N % PD][i];
#pragma unroll
            for (int t = 1; t < WP; ++t) acc = comb<T, OP>(acc, xq[N % PD][(i - t + WP) % WP]);
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
};

template <class T, int OP, int WP>
__global__ void __launch_bounds__(kWaveThreads) wave_tier_kernel(RunArgs A, WaveLayout wl)
{
    const Geom& g = A.g;
    const TierDesc& td = A.tiers[0];
    const uint32_t lane = threadIdx.x;
    const uint32_t wshift = td.dlo - wl.slot_shift;            // wavefronts per scenario = 2^wshift
    const uint32_t sv = blockIdx.x >> wshift;                  // scenario, or S + retry entry
    const uint32_t top0 = (1u << td.dlo) - 1u;
    const uint32_t cone_w = (blockIdx.x & ((1u << wshift) - 1u)) << wl.slot_shift;
    if (top0 + cone_w >= g.M) return;                          // no such rows

    // lane -> (subtree slot, value index e)
    const uint32_t slot = lane / wl.ne;
    const uint32_t e = lane - slot * wl.ne;
    const bool active = lane < wl.nact;
    const uint32_t cone = cone_w + (active ? slot : 0u);
    const uint32_t rs = top0 + cone;                           // top row of the lane's subtree
    const bool exists = active && rs < g.M;

    // shape of the lane's subtree: complete with or without the bottom level, or ragged
    const uint32_t first_leaf = ((rs + 1u) << kWaveH) - 1u;
    const uint32_t last_leaf = ((rs + 2u) << kWaveH) - 2u;
    const bool bottom = last_leaf < g.M;
    auto in_tree = [&](uint32_t jr) -> bool {                  // is row jr inside the lane's subtree?
        if (jr == kNoRank) return false;
        const uint32_t d = ilog2(jr + 1u);
        if (d < td.dlo || d > td.dlo + uint32_t(kWaveH)) return false;
        return ((jr + 1u) >> (d - td.dlo)) - 1u == rs;
    };
    bool handover = !bottom && first_leaf < g.M;               // ragged bottom level
    if (g.a > 1 && in_tree(g.M - 1u)) handover = true;         // the short last group (the root is a member)

    uint32_t s = sv, root = 0, status = kStOk, frank = kNoRank;
    unsigned char* wsS;
    const uint32_t F = g.f > 0 ? g.f : 1;
    if (sv < A.S) {
        status = A.status[s];
        if (A.attempts) root = A.attempts[s];                  // roots tried; the last one is alive
        else if (A.root) root = A.root[s];
        if (lane < g.f) frank = A.fail_rank[size_t(s) * F + lane];
        if (A.attempts) root = root > 0 ? root - 1u : 0u;
        wsS = A.ws + size_t(s) * A.ws_stride;
    } else {
        const uint32_t kk = sv - A.S;
        if (kk >= *A.retry_count) return;
        s = __builtin_amdgcn_readfirstlane(A.retry_list[2u * kk]);
        root = A.retry_list[2u * kk + 1u];
        if (lane < g.f) frank = A.fail_rank[size_t(s) * F + lane];
        wsS = A.retry_ws + size_t(kk) * A.ws_stride;
    }
    status = __builtin_amdgcn_readfirstlane(status);
    root = __builtin_amdgcn_readfirstlane(root);
    if (status == kStBadFailureSet) return;
    // rows of the listed processes, and of the process that carries the root's number
    {
        uint32_t frow = kNoRank;
        if (frank != kNoRank) {
            const uint32_t vr = relabel(frank, root);
            frow = vr == 0 ? (g.a > 1 ? g.M - 1u : kNoRank) : fdiv(vr - 1u, g.divW);
        }
        for (uint32_t q = 0; q < g.f; ++q)
            if (in_tree(uint32_t(__builtin_amdgcn_readlane(int(frow), int(q))))) handover = true;
        if (root != 0 && in_tree(fdiv(root - 1u, g.divW))) handover = true;
    }
    if (exists && handover && e == 0) {
        // not for this kernel: the general (LDS tile) kernel runs this subtree
        const uint32_t n = atomicAdd(A.fix_count, 1u);
        A.fix_list[2u * n] = sv;
        A.fix_list[2u * n + 1u] = cone;
    }
    const bool mine = exists && !handover;
    const bool any_bottom = __ballot(mine && bottom) != 0ull;  // else no lane here has the deepest level

    const unsigned char* pay = A.payload + size_t(s) * A.scen_stride_bytes;
    const unsigned char* bk[WP];
#pragma unroll
    for (int k = 0; k < WP; ++k) bk[k] = pay + size_t(k) * g.EB;
    for (uint32_t pass = 0; pass < wl.passes; ++pass) {
        const uint32_t ecol = pass * wl.ne + e;
        if (mine && ecol < g.E) {
            T out[WP];
            if (any_bottom) {
                SubtreeWalk<T, OP, WP, kWaveH> w(g, bk, rs, ecol, bottom);
                w.run();
#pragma unroll
                for (int k = 0; k < WP; ++k) out[k] = w.cur[k];
            } else {
                SubtreeWalk<T, OP, WP, kWaveH - 1> w(g, bk, rs, ecol, true);
                w.run();
#pragma unroll
                for (int k = 0; k < WP; ++k) out[k] = w.cur[k];
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
    // every process of the rows folded here sent all its messages
    if (A.msgs) {
        const unsigned long long rows =
            (unsigned long long)__popcll(__ballot(mine && e == 0 && bottom)) * ((2u << kWaveH) - 1u) +
            (unsigned long long)__popcll(__ballot(mine && e == 0 && !bottom)) * ((1u << kWaveH) - 1u);
        if (lane == 0 && rows != 0) {
            atomicAdd(&A.msgs[size_t(s) * A.nmsg + 0], rows * g.W * (g.W - 1u));
            atomicAdd(&A.msgs[size_t(s) * A.nmsg + 1], rows * g.W);
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
        hipLaunchKernelGGL((wave_tier_kernel<T, OP, WP>), dim3(grid), dim3(kWaveThreads), 0, st, A, wl); \
        return hipGetLastError();                                                                   \
    }                                                                                               \
    hipError_t launch_wave_##NAME(const RunArgs& A, const WaveLayout& wl, uint32_t grid, hipStream_t st) \
    {                                                                                               \
        switch (A.g.W) {          /* the widths of wave_width_ok() */                               \
            case 2: return wave_wp_##NAME<2>(A, wl, grid, st);                                      \
            case 3: return wave_wp_##NAME<3>(A, wl, grid, st);                                      \
            case 4: return wave_wp_##NAME<4>(A, wl, grid, st);                                      \
            case 5: return wave_wp_##NAME<5>(A, wl, grid, st);                                      \
            case 9: return wave_wp_##NAME<9>(A, wl, grid, st);                                      \
            default: return hipErrorInvalidValue;                                                   \
        }                                                                                           \
    }

}  // namespace ftred

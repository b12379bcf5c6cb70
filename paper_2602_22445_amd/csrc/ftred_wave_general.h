// Deepest tier, subtrees with listed processes: the register walk of
// ftred_wave.h with the failure handling of the tile kernel.
//
// A lane owns (list entry, value index): the entry names a subtree of height
// kWaveH of one scenario (or retry entry) that the plain register kernel leaves
// out: some members are listed as failed, or it holds the last row, which may be
// short (the root is then a member of its up-correction group, section
// "Up-Correction") and may end an incomplete bottom level.  The walk is the same
// post-order walk in registers; in addition every row carries a word of sent and
// failed bits, as in the tile kernel (process_item), and the additions are
// predicated:
//   - up-correction (Algorithm "Up-correction"): member i folds the input of
//     member w, due in round t = (i - w) mod W, iff w still sends in round t;
//   - tree phase (Algorithm "reduce at non-roots"): a member adds a child's message
//     iff the child sent one, and sets its failed bit if a child's message is
//     missing or carries the bit (section "Failure information", third scheme).
// What a row needs to know about its listed members (rounds in which each member
// still sends, who sends a tree message) is written once per entry into a small
// LDS table indexed by the row's position in the subtree, so a visit costs one LDS
// read.  The lanes of a wavefront may belong to different scenarios: everything
// about the scenario is per lane here.
//
// Not for this kernel (they stay with the tile kernel): every listed subtree when
// the lists of failed processes are asked for.  The last row is always on the
// deepest level of its subtree (the tree has at least kWaveH + 2 levels), so only
// the visits of that level know about short or missing rows.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ftred_geom.h"
#include "ftred_kernels.h"
#include "ftred_wave.h"

namespace ftred {

// per (entry, row of its subtree): 4 bits per member = up-correction rounds in which the member still
// sends; bit k of sent = member k sends its tree message
struct RowInfo {
    uint32_t tl_lo, tl_hi, sent;
    uint32_t gs;             // members of the row's up-correction group (the root included, if it is one)
};

template <class T, int OP, int WP, int HH>
struct GeneralWalk {
    static constexpr int PD = 2;                   // rows requested ahead
    static constexpr int NR = (2 << HH) - 1;
    const Geom& g;
    const unsigned char* pay;      // this lane's scenario
    const RowInfo* info;           // LDS: this lane's entry, by position in the subtree
    uint32_t rs, ecol, root;
    bool count;
    T* vroot;                      // where the root's value after its up-correction goes (this lane's value index)
    uint32_t jx, kx;               // the relabelled rank (jx = kNoRank: the root is process 0)
    T x0;
    T xq[PD][WP];
    T st[HH + 1][WP];
    T cur[WP];
    uint32_t st_meta[HH + 1], cur_meta;      // bits 0..15 sent, 16..31 failed bit, per member
    uint32_t uc_cnt, tree_cnt;               // messages sent by the rows of this subtree (lane with count only)

    __device__ __forceinline__ GeneralWalk(const Geom& g_, const unsigned char* pay_, const RowInfo* info_, uint32_t rs_,
                                           uint32_t ecol_, bool count_, uint32_t root_, T* vroot_)
        : g(g_), pay(pay_), info(info_), rs(rs_), ecol(ecol_), root(root_), count(count_), vroot(vroot_)
    {
        jx = kNoRank; kx = 0; x0 = T(0);
        if (root != 0) {
            jx = fdiv(root - 1u, g.divW);
            kx = root - 1u - jx * g.W;
            x0 = *reinterpret_cast<const T*>(pay + size_t(ecol) * g.esz);
        }
        uc_cnt = tree_cnt = 0;
        cur_meta = 0;
    }

    template <int N>
    __device__ __forceinline__ void issue()
    {
        constexpr int li = cx_postorder(N, HH);
        constexpr int l = cx_ilog2(li + 1);
        const uint32_t j = ((rs + 1u) << l) - 1u + uint32_t(li - ((1 << l) - 1));
        const uint32_t off = ((1u + j * g.W) * g.E + ecol) * g.esz;
        const uint32_t safe = ecol * g.esz;                     // process 0: a valid address for what does not exist
        if constexpr (l < HH) {
#pragma unroll
            for (int k = 0; k < WP; ++k) xq[N % PD][k] = *reinterpret_cast<const T*>(pay + size_t(k) * g.EB + off);
        } else {
            // the deepest level: rows may be missing, the last row may be short and hold the root as member a - 1
            const bool ex = j < g.M, last = j == g.M - 1u;
            const uint32_t nk = last ? g.nlast : g.W;
            const uint32_t off_root = root * g.EB + safe;
#pragma unroll
            for (int k = 0; k < WP; ++k) {
                uint32_t o = uint32_t(k) * g.EB + off;
                if (!ex || uint32_t(k) >= nk) o = (last && g.a > 1 && uint32_t(k) == g.a - 1u) ? off_root : safe;
                xq[N % PD][k] = *reinterpret_cast<const T*>(pay + o);
            }
        }
    }

    template <int N>
    __device__ __forceinline__ void visit()
    {
        constexpr int li = cx_postorder(N, HH);
        constexpr int l = cx_ilog2(li + 1);
        constexpr uint32_t mask = (1u << WP) - 1u;
#pragma unroll
        for (int k = 0; k < WP; ++k) asm volatile("" : "+v"(xq[N % PD][k]) : : "memory");
        // what depends on the row is worked out at its visit, not for all rows ahead of the walk (registers)
        asm volatile("" : "+v"(rs));
        const uint32_t j = ((rs + 1u) << l) - 1u + uint32_t(li - ((1 << l) - 1));
        const bool here = j == jx;
#pragma unroll
        for (int k = 0; k < WP; ++k) xq[N % PD][k] = (here && kx == uint32_t(k)) ? x0 : xq[N % PD][k];
        const RowInfo ri = info[li];
        const unsigned long long tl = (unsigned long long)ri.tl_lo | ((unsigned long long)ri.tl_hi << 32);
        const uint32_t sent = ri.sent & mask;

        // up-correction: in round t = (i - w) mod gs member i receives the input of member w iff w still sends
        // then; gs = W except in a short last row, which is on the deepest level
        const uint32_t gs = l < HH ? uint32_t(WP) : ri.gs;
        T v[WP];
#pragma unroll
        for (int i = 0; i < WP; ++i) {
            T acc = xq[N % PD][i];
#pragma unroll
            for (int w = i - 1; w >= 0; --w) {                 // rounds 1 .. i
                const T sum = comb<T, OP>(acc, xq[N % PD][w]);
                acc = exchange_round(uint32_t(w), uint32_t(i), gs) <= uint32_t((tl >> (4 * w)) & 15ull) ? sum : acc;
            }
#pragma unroll
            for (int w = WP - 1; w > i; --w) {                 // rounds i + 1 .. gs - 1
                const T sum = comb<T, OP>(acc, xq[N % PD][w]);
                const uint32_t t = exchange_round(uint32_t(w), uint32_t(i), gs);
                acc = (uint32_t(w) < gs && t <= uint32_t((tl >> (4 * w)) & 15ull)) ? sum : acc;
            }
            v[i] = acc;
        }
        if constexpr (l == HH) {
            // the root's value after its up-correction: member a - 1 of the short last row
            if (j == g.M - 1u && g.a > 1) {
                T vr = T(0);
#pragma unroll
                for (int k = 0; k < WP; ++k) vr = uint32_t(k) == g.a - 1u ? v[k] : vr;
                *vroot = vr;
            }
        }
        if constexpr (N + PD < NR) issue<N + PD>();
        // tree phase: the lower-numbered child's message first; on the level above the deepest one a child row
        // may be missing (nothing to add, nothing to report) or short
        uint32_t flag = 0;
        if constexpr (l < HH) {
            const uint32_t cl = st_meta[l + 1], cr = cur_meta;
            bool exl = true, exr = true;
            uint32_t ml = mask, mr = mask;
            if constexpr (l == HH - 1) {
                const uint32_t jl = 2u * j + 1u, jr = 2u * j + 2u;
                exl = jl < g.M; exr = jr < g.M;
                ml = jl == g.M - 1u ? (1u << g.nlast) - 1u : mask;
                mr = jr == g.M - 1u ? (1u << g.nlast) - 1u : mask;
            }
#pragma unroll
            for (int k = 0; k < WP; ++k) {
                const T a = comb<T, OP>(v[k], st[l + 1][k]);
                v[k] = (exl && ((cl >> k) & ml >> k & 1u)) ? a : v[k];
                const T b = comb<T, OP>(v[k], cur[k]);
                v[k] = (exr && ((cr >> k) & mr >> k & 1u)) ? b : v[k];
            }
            flag = (exl ? ((cl >> 16) | ~cl) & ml : 0u) | (exr ? ((cr >> 16) | ~cr) & mr : 0u);
        }
        const uint32_t meta = sent | (flag << 16);
        if (count && j < g.M) {
            uint32_t c = 0;
#pragma unroll
            for (int w = 0; w < WP; ++w) c += uint32_t(w) < gs ? uint32_t((tl >> (4 * w)) & 15ull) : 0u;
            uc_cnt += c;
            tree_cnt += uint32_t(__popc(sent));
        }
        if constexpr (li != 0 && (li & 1)) {
#pragma unroll
            for (int k = 0; k < WP; ++k) st[l][k] = v[k];
            st_meta[l] = meta;
        } else {
#pragma unroll
            for (int k = 0; k < WP; ++k) cur[k] = v[k];
            cur_meta = meta;
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

// The entries first .. first + 2^slot_shift - 1 of one of the two parts of the list (front: entries without
// rows on the deepest level, from the front of the list; else those with such rows, from its back; n = entries
// of that part), one per slot of the wavefront.
template <class T, int OP, int WP>
__device__ __forceinline__ void wave_list_entries(const RunArgs& A, const WaveLayout& wl, RowInfo* rinfo, bool front,
                                                  uint32_t first, uint32_t n)
{
    const Geom& g = A.g;
    const TierDesc& td = A.tiers[0];
    const uint32_t lane = threadIdx.x;
    const uint32_t slot = lane / wl.ne;
    const uint32_t e = lane - slot * wl.ne;
    const uint32_t at = first + slot;
    const bool valid = lane < wl.nact && at < n;
    const uint32_t idx = front ? at : A.wfix_cap - 1u - at;
    const uint32_t top0 = (1u << td.dlo) - 1u;
    const uint32_t F = g.f > 0 ? g.f : 1;

    // the entry: (scenario or S + retry entry, subtree, scenario, root)
    const vec16_t w = reinterpret_cast<const vec16_t*>(A.wfix_list)[valid ? idx : 0u];
    const uint32_t sv = w.x, cone = w.y, s = w.z, root = w.w;
    const bool discard = sv >= A.S;
    const uint32_t base = (discard || A.attempts) ? root * g.Ratt : 0u;
    unsigned char* wsS = discard ? A.retry_ws + size_t(sv - A.S) * A.ws_stride : A.ws + size_t(s) * A.ws_stride;
    const unsigned char* pay = A.payload + size_t(s) * A.scen_stride_bytes;
    const uint32_t rs = top0 + cone;
    const bool deep = (((rs + 1u) << kWaveH) - 1u) < g.M;       // the entry has rows on the deepest level

    // the rows of the entry: nobody listed ...
    RowInfo* mine = rinfo + size_t(slot) * kWaveRows;
    if (valid) {
        for (uint32_t li = e; li < kWaveRows; li += wl.ne) {
            const uint32_t d = ilog2(li + 1u);
            const uint32_t j = (rs << d) + li;
            const bool last = j == g.M - 1u;
            const uint32_t gs = (last && g.a > 1) ? g.a : g.W;
            const uint32_t nk = last ? g.nlast : g.W;
            const unsigned long long all = 0x1111111111111111ull * (unsigned long long)(gs - 1u);
            RowInfo d0;
            d0.tl_lo = uint32_t(all); d0.tl_hi = uint32_t(all >> 32); d0.sent = (1u << nk) - 1u; d0.gs = gs;
            mine[li] = d0;
        }
    }
    __syncthreads();
    // ... then the listed ones, by the first lane of the entry
    if (valid && e == 0) {
        for (uint32_t q = 0; q < g.f; ++q) {
            const uint32_t rank = A.fail_rank[size_t(s) * F + q];
            if (rank == kNoRank) continue;
            const uint32_t vr = relabel(rank, root);
            uint32_t j, k, gs;
            bool tree = false;
            const uint32_t fr = A.fail_round[size_t(s) * F + q];
            if (vr == 0) {                                      // the root: member a - 1 of the short last row, if any
                if (g.a <= 1) continue;
                j = g.M - 1u; k = g.a - 1u; gs = g.a;
            } else {
                j = fdiv(vr - 1u, g.divW);
                k = vr - 1u - j * g.W;
                gs = group_size(g, j);
                tree = alive_at(fr, base + tree_send_round(g, k, j));
            }
            if (subtree_of_row(j, td.dlo) != cone) continue;
            const uint32_t li = j - (rs << (ilog2(j + 1u) - td.dlo));        // position inside the subtree (heap order)
            const uint32_t done = fr > base + 1u ? fr - base - 1u : 0u;      // up-correction rounds it still sends in
            const uint32_t uc = done < gs - 1u ? done : gs - 1u;
            RowInfo d0 = mine[li];
            unsigned long long tl = (unsigned long long)d0.tl_lo | ((unsigned long long)d0.tl_hi << 32);
            tl = (tl & ~(15ull << (4u * k))) | ((unsigned long long)uc << (4u * k));
            d0.tl_lo = uint32_t(tl); d0.tl_hi = uint32_t(tl >> 32);
            if (!tree) d0.sent &= ~(1u << k);
            mine[li] = d0;
        }
    }
    __syncthreads();

    const bool any_deep = __ballot(valid && deep) != 0ull;
    uint32_t uc_cnt = 0, tree_cnt = 0;
    // the blocks of value indices of an entry are workgroups of their own (grid dimension y)
    for (uint32_t pass = blockIdx.y; pass < wl.passes; pass += gridDim.y) {
        const uint32_t ecol = pass * wl.ne + e;
        if (valid && ecol < g.E) {
            T out[WP];
            uint32_t meta;
            T* vroot = reinterpret_cast<T*>(wsS + A.vroot_off) + ecol;
            if (any_deep) {
                GeneralWalk<T, OP, WP, kWaveH> gw(g, pay, mine, rs, ecol, ecol == 0, root, vroot);
                gw.run();
#pragma unroll
                for (int k = 0; k < WP; ++k) out[k] = gw.cur[k];
                meta = gw.cur_meta; uc_cnt += gw.uc_cnt; tree_cnt += gw.tree_cnt;
            } else {
                GeneralWalk<T, OP, WP, kWaveH - 1> gw(g, pay, mine, rs, ecol, ecol == 0, root, vroot);
                gw.run();
#pragma unroll
                for (int k = 0; k < WP; ++k) out[k] = gw.cur[k];
                meta = gw.cur_meta; uc_cnt += gw.uc_cnt; tree_cnt += gw.tree_cnt;
            }
            unsigned char* dst = wsS + td.out_off + size_t(cone) * g.RB + size_t(ecol) * g.esz;
#pragma unroll
            for (int k = 0; k < WP; ++k) *reinterpret_cast<T*>(dst + size_t(k) * g.EB) = out[k];
            if (ecol == 0) reinterpret_cast<uint32_t*>(wsS + td.out_meta_off)[cone] = meta;
        }
    }
    if (A.msgs && valid && e == 0) {
        if (uc_cnt) atomicAdd(&A.msgs[size_t(s) * A.nmsg + 0], (unsigned long long)uc_cnt);
        if (tree_cnt) atomicAdd(&A.msgs[size_t(s) * A.nmsg + 1], (unsigned long long)tree_cnt);
    }
}

// One wavefront per workgroup; lanes = (entry slot, value index) as in the register
// kernel, an entry per slot.  Workgroups from the front of the grid take the front
// part of the list, workgroups from its back the back part (so a wavefront walks
// subtrees of one height).  Dynamic LDS: 2^slot_shift * kWaveRows RowInfo.
// The walk is a chain of loads that wait for each other: for the narrower groups the registers are held
// to what lets two wavefronts share a SIMD.
template <class T, int OP, int WP>
__global__ void __launch_bounds__(kWaveThreads) __attribute__((amdgpu_waves_per_eu(WP <= 5 ? 2 : 1)))
wave_list_kernel(RunArgs A, WaveLayout wl)
{
    extern __shared__ __align__(16) unsigned char smem[];
    RowInfo* rinfo = reinterpret_cast<RowInfo*>(smem);
    const uint32_t nslots = 1u << wl.slot_shift;
    const uint32_t n_front = A.wfix_count[0], n_back = A.wfix_count[1];
    const uint32_t bb = gridDim.x - 1u - blockIdx.x;
    if (blockIdx.x * nslots < n_front) wave_list_entries<T, OP, WP>(A, wl, rinfo, true, blockIdx.x * nslots, n_front);
    if (bb * nslots < n_back) {
        __syncthreads();          // the table is used again
        wave_list_entries<T, OP, WP>(A, wl, rinfo, false, bb * nslots, n_back);
    }
}

#define FTRED_DECLARE_WAVE_LIST_LAUNCHER(NAME) \
    hipError_t launch_wave_list_##NAME(const RunArgs& A, const WaveLayout& wl, uint32_t grid, uint32_t lds, hipStream_t st);

FTRED_DECLARE_WAVE_LIST_LAUNCHER(i64_sum)
FTRED_DECLARE_WAVE_LIST_LAUNCHER(i64_bor)
FTRED_DECLARE_WAVE_LIST_LAUNCHER(u32_sum)
FTRED_DECLARE_WAVE_LIST_LAUNCHER(u32_bor)
FTRED_DECLARE_WAVE_LIST_LAUNCHER(f64_sum)

#define FTRED_DEFINE_WAVE_LIST_LAUNCHER(NAME, T, OP)                                                \
    template <int WP>                                                                               \
    static hipError_t wave_list_wp_##NAME(const RunArgs& A, const WaveLayout& wl, uint32_t grid, uint32_t lds, hipStream_t st) \
    {                                                                                               \
        hipLaunchKernelGGL((wave_list_kernel<T, OP, WP>), dim3(grid, wl.passes < 65535u ? wl.passes : 65535u),  \
                           dim3(kWaveThreads), lds, st, A, wl);                                       \
        return hipGetLastError();                                                                   \
    }                                                                                               \
    hipError_t launch_wave_list_##NAME(const RunArgs& A, const WaveLayout& wl, uint32_t grid, uint32_t lds, hipStream_t st) \
    {                                                                                               \
        FTRED_WAVE_WIDTH_SWITCH(A.g.W, wave_list_wp_##NAME, A, wl, grid, lds, st)                   \
    }

}  // namespace ftred

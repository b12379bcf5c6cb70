// The whole tree phase of one scenario in one workgroup: the register walk of
// ftred_wave.h for the deepest tier, then the levels above it and the root's
// choice out of LDS, in the same launch.
//
// A workgroup of nw <= 4 wavefronts owns one scenario (or retry entry).  Each
// wavefront walks through its groups of sibling subtrees exactly as in
// wave_tier_kernel (one lane per subtree and value index, no cross-lane traffic),
// but the top rows of the subtrees stay in LDS: [subtree][member][value index],
// 2^dlo rows.  The subtrees that the plain walk leaves out (listed processes, the
// short last group, a ragged bottom: at most f + 1 per scenario) were folded by
// the list kernel in an EARLIER launch; their top rows come in from the scratch
// area.  After one barrier the rows of depths dlo-1 .. 0 are folded level by
// level: one thread per (row, value index) loads the W inputs of its row straight
// from HBM (requested for all levels at once, right after the walk, when the
// walk's registers are free), forms the up-correction values in round order
// (Algorithm "Up-correction"), adds the messages of the two children rows out of
// LDS (Algorithm "reduce at non-roots"; sent and failed bits per member, section
// "Failure information", third scheme) and, after a barrier, puts its messages
// where the level above finds them.  The last level leaves the messages of the
// root's children, and the root takes its choice (Algorithm "reduce at the root").
// Nothing but the result leaves the workgroup: no top rows go through HBM, and no
// further launch is needed for the levels above the deepest tier.
//
// Used when the levels above the deepest tier are few enough: 2^dlo top rows fit
// the LDS tile and (2^dlo - 1) * E items are at most four per thread.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>

#include "ftred_geom.h"
#include "ftred_kernels.h"
#include "ftred_wave.h"

namespace ftred {

constexpr uint32_t kFusedMaxWaves = 4;
constexpr int kFusedItems = 4;                       // (row, value index) items of the upper levels per thread

struct FusedLayout {
    uint32_t ne, slot_shift, nact;   // lanes of a wavefront = 2^slot_shift sibling subtrees x ne value indices
    uint32_t group_shift;            // a wavefront walks through 2^group_shift groups of subtrees
    uint32_t wshift;                 // wavefronts per workgroup = 2^wshift
    uint32_t passes;                 // blocks of ne value indices: a workgroup per scenario and block
    FastDiv div_passes;
    uint32_t one;                    // always 1: trip count of the loop around the walk (see the kernel)
    FastDiv div_ne;
    uint32_t dp;                     // a workgroup folds the part of the tree below ONE row of depth dp (2^dp parts per
                                     // scenario; 0: the whole tree and the root's choice)
    uint32_t ok;                     // the plan can use the fused kernel
};

// most LDS for the top rows of one scenario's subtrees (one block of value indices): three workgroups per CU for
// the narrow groups (three wavefronts per SIMD), two for the wider ones
inline uint32_t fused_tile_bytes(uint32_t W) { return W <= 5u ? 48u * 1024u : 72u * 1024u; }

inline FusedLayout make_fused_layout(const Geom& g, uint32_t dlo_tree, uint32_t dp = 0)
{
    FusedLayout f;
    memset(&f, 0, sizeof(f));
    f.dp = dp;
    const uint32_t dlo = dlo_tree - dp;              // levels of a part above its subtrees' top rows
    // the block of value indices: as many as a wavefront has lanes for, fewer where the top rows of a wider block
    // do not fit the tile, but at least a 128-byte line of every process's payload (or all of it)
    for (uint32_t ne = g.E < 64u ? g.E : 64u; ne >= 1u; ne /= 2u) {
        uint32_t slots = 64u / ne, sh = 0;
        while ((2u << sh) <= slots && sh < dlo) ++sh;
        f.ne = ne; f.slot_shift = sh; f.nact = (1u << sh) * ne;
        f.passes = (g.E + ne - 1u) / ne;
        f.div_passes = make_fastdiv(f.passes);
        f.one = 1;
        f.div_ne = make_fastdiv(ne);
        const uint32_t rest = dlo - sh;               // log2 of the groups of subtrees per scenario
        f.group_shift = rest > 2u ? (rest - 2u < 2u ? rest - 2u : 2u) : 0u;
        f.wshift = rest - f.group_shift;
        const uint64_t items = ((uint64_t(1) << dlo) - 1u) * ne;
        f.ok = ((1u << f.wshift) <= kFusedMaxWaves &&
                ((uint64_t(g.W) * ne * g.esz) << dlo) <= fused_tile_bytes(g.W) &&
                items <= uint64_t(kFusedItems) * 64u * (1u << f.wshift)) ? 1u : 0u;
        if (f.ok || (ne / 2u) * g.esz < 128u || ne % 2u != 0u) break;
    }
    return f;
}

// dynamic LDS: failure table, the top rows (one block of value indices), one word of sent / failed bits and one
// "folded here" word per subtree
inline uint32_t fused_lds_bytes(const Geom& g, const FusedLayout& fl, uint32_t dlo)
{
    return uint32_t(sizeof(FailTab)) + ((g.W * fl.ne * g.esz) << (dlo - fl.dp)) + (8u << (dlo - fl.dp));
}

// One (row, value index) item of the levels above the deepest tier.  The row is complete (W members, the root is
// not in its group: the last row lies on the deepest level of the tree) and so are its two children rows.
// x: the inputs of the row's members; c0, c1: the messages of the children rows in LDS (member stride ms);
// cm0, cm1: their sent (bits 0..15) and failed (16..31) bits.  Leaves the members' tree messages in x.
template <class T, int OP, int WP>
__device__ __forceinline__ uint32_t fused_item(const FailTab& ft, bool check_fail, uint32_t j, T (&x)[WP],
                                               const T* c0, const T* c1, uint32_t ms, uint32_t cm0, uint32_t cm1,
                                               bool count, uint32_t& uc_cnt, uint32_t& tree_cnt)
{
    constexpr uint32_t mask = (1u << WP) - 1u;
    // failures of this row: tl = packed 4-bit "rounds in which member w still sends"
    unsigned long long tl = 0x1111111111111111ull * (unsigned long long)(WP - 1);
    uint32_t sent = mask;
    bool rowfail = false;
    if (check_fail) {
        for (uint32_t q = 0; q < ft.n; ++q) {
            if (ft.row[q] == j) {
                rowfail = true;
                const uint32_t i4 = 4u * ft.idx[q];
                tl = (tl & ~(15ull << i4)) | ((unsigned long long)ft.uc[q] << i4);
                if (!ft.tree[q]) sent &= ~(1u << ft.idx[q]);
            }
        }
    }
    // up-correction: member i folds, in round order t = 1..W-1, the input of member (i - t) mod W, if that member
    // still sends in round t
    T v[WP];
    if (!rowfail) {
#pragma unroll
        for (int i = 0; i < WP; ++i) {
            T acc = x[i];
#pragma unroll
            for (int t = 1; t < WP; ++t) acc = comb<T, OP>(acc, x[exchange_source(uint32_t(i), uint32_t(t), uint32_t(WP))]);
            v[i] = acc;
        }
    } else {
#pragma unroll
        for (int i = 0; i < WP; ++i) {
            T acc = x[i];
#pragma unroll
            for (int t = 1; t < WP; ++t) {
                const int w = int(exchange_source(uint32_t(i), uint32_t(t), uint32_t(WP)));
                if (uint32_t(t) <= uint32_t((tl >> (4 * w)) & 15ull)) acc = comb<T, OP>(acc, x[w]);
            }
            v[i] = acc;
        }
    }
    // tree phase: the lower-numbered child's message first; a missing message or one that carries the failed bit
    // sets the failed bit
    if ((cm0 & mask) == mask && (cm1 & mask) == mask) {
#pragma unroll
        for (int k = 0; k < WP; ++k) v[k] = comb<T, OP>(comb<T, OP>(v[k], c0[k * ms]), c1[k * ms]);
    } else {
#pragma unroll
        for (int k = 0; k < WP; ++k) {
            if ((cm0 >> k) & 1u) v[k] = comb<T, OP>(v[k], c0[k * ms]);
            if ((cm1 >> k) & 1u) v[k] = comb<T, OP>(v[k], c1[k * ms]);
        }
    }
    const uint32_t flag = (((cm0 >> 16) | ~cm0) | ((cm1 >> 16) | ~cm1)) & mask;
#pragma unroll
    for (int k = 0; k < WP; ++k) x[k] = v[k];
    if (count) {
        uint32_t c = 0;
#pragma unroll
        for (int w = 0; w < WP; ++w) c += uint32_t((tl >> (4 * w)) & 15ull);
        uc_cnt += c;
        tree_cnt += uint32_t(__popc(sent));
    }
    return sent | (flag << 16);
}

template <class T, int OP, int WP>
__global__ void __launch_bounds__(kFusedMaxWaves * 64) __attribute__((amdgpu_waves_per_eu(WP <= 5 ? 3 : 2))) fused_tree_kernel(RunArgs A, FusedLayout fl)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const Geom& g = A.g;
    const TierDesc& td = A.tiers[0];
    const uint32_t dlo = td.dlo - fl.dp;             // levels of the workgroup's part above its subtrees' top rows
    const uint32_t tid = threadIdx.x, nthr = blockDim.x;
    const uint32_t lane = tid & 63u;
    const uint32_t wid = __builtin_amdgcn_readfirstlane(tid >> 6);     // the same in all lanes: addresses of rows stay scalar
    const uint32_t ncones = 1u << dlo;
    const uint32_t ne = fl.ne, REl = g.W * ne;       // a row of the tile: W members x ne value indices of the block
    const uint32_t top0 = (1u << td.dlo) - 1u;       // first row of the subtrees' top level in the whole tree
    FailTab& ft = *reinterpret_cast<FailTab*>(smem);
    T* tile = reinterpret_cast<T*>(smem + sizeof(FailTab));
    uint32_t* lmeta = reinterpret_cast<uint32_t*>(smem + sizeof(FailTab) + (size_t(REl) * g.esz << dlo));
    uint32_t* folded = lmeta + ncones;

    // ---- which scenario, which block of value indices, which root
    // the workgroup's part of the tree: the rows below row `part` of depth fl.dp (the whole tree if fl.dp == 0)
    const uint32_t part = blockIdx.x & ((1u << fl.dp) - 1u);
    const uint32_t cone0 = part << dlo;              // its first subtree
    uint32_t sv = blockIdx.x >> fl.dp, pass = 0;     // scenario, or S + retry entry
    if (fl.passes > 1u) {
        const uint32_t b = sv;
        sv = fdiv(b, fl.div_passes);
        pass = b - sv * fl.passes;
    }
    uint32_t s = sv, root = 0, base = 0;
    bool discard = false;
    unsigned char* wsS;
    if (sv < A.S) {
        if (A.status[s] == kStBadFailureSet) return;
        if (A.attempts) {
            root = A.attempts[s] - 1u;               // roots tried; the last one is alive
            base = root * g.Ratt;
        } else if (A.root) {
            root = A.root[s];
        }
        wsS = A.ws + size_t(s) * A.ws_stride;
    } else {
        // an attempt whose root had failed beforehand: messages are sent, nothing is delivered
        const uint32_t kk = sv - A.S;
        if (kk >= *A.retry_count) return;
        s = A.retry_list[2u * kk];
        root = A.retry_list[2u * kk + 1u];
        base = root * g.Ratt;
        discard = true;
        wsS = A.retry_ws + size_t(kk) * A.ws_stride;
    }
    s = __builtin_amdgcn_readfirstlane(s);
    root = __builtin_amdgcn_readfirstlane(root);
    const unsigned char* pay = A.payload + size_t(s) * A.scen_stride_bytes;
    const uint32_t F = g.f > 0 ? g.f : 1;

    load_failtab(ft, g, A.fail_rank, A.fail_round, s, root, base);
    // lane -> (subtree slot, value index of the block); the subtrees that the list kernel folded, one per lane
    const uint32_t slot = lane / ne;
    const uint32_t e = lane - slot * ne;
    const bool active = lane < fl.nact;
    const uint32_t listed = lane < g.f ? A.fail_rank[size_t(s) * F + lane] : kNoRank;
    const uint32_t special = subtree_of_row(special_row_of_lane(g, td.dlo, listed, root, lane), td.dlo) - cone0;
    const unsigned char* bk[WP];
#pragma unroll
    for (int k = 0; k < WP; ++k) bk[k] = pay + size_t(k) * g.EB;
    uint32_t uc_cnt = 0, tree_cnt = 0;
    uint32_t st = kStOk;

    // The workgroup folds the whole tree for ITS block of ne value indices (one block unless a process holds more
    // than 64 values; the blocks of a scenario are workgroups of their own), the top rows in LDS.  The walk itself
    // sits in a loop whose trip count (one) the compiler does not know, with a value index that depends on the
    // trip: as straight-line code, or in a loop whose body does not change, the loads of a whole walk are
    // requested ahead of it and the kernel needs 300 to 500 registers instead of 160.
    {
        const uint32_t ecol_p = pass * ne + e;
        for (uint32_t c = tid; c < ncones; c += nthr) folded[c] = 0u;
        __syncthreads();                              // also: the failure table is there

        // ---- the deepest tier: every wavefront walks through its groups of subtrees (as wave_tier_kernel does)
        for (uint32_t gi = 0; gi < (1u << fl.group_shift); ++gi) {
            // the groups of a wavefront lie a stride of wavefronts apart: side by side run wavefronts that read
            // rows side by side
            const uint32_t cone_w = (wid + (gi << fl.wshift)) << fl.slot_shift;      // within the part
            if (top0 + cone0 + cone_w >= g.M) break;
            const uint32_t cone = cone_w + (active ? slot : 0u);
            const uint32_t rs = top0 + cone0 + cone;               // top row of the lane's subtree
            const bool exists = active && rs < g.M;
            const uint32_t last_leaf = ((rs + 2u) << kWaveH) - 2u;
            const bool bottom = last_leaf < g.M;                   // complete with the bottom level (a ragged one is listed)
            bool handover = false;                                 // a listed subtree: folded by the list kernel
            unsigned long long hits = __ballot(special - cone_w < (1u << fl.slot_shift));
            while (hits != 0ull) {
                const int en = __ffsll(hits) - 1;
                hits &= hits - 1ull;
                if (uint32_t(__builtin_amdgcn_readlane(int(special), en)) == cone) handover = true;
            }
            const bool mine = exists && !handover;
            const bool any_bottom = __ballot(mine && bottom) != 0ull;
            for (uint32_t rep = 0; rep < fl.one; ++rep) {          // one trip: see above
            const uint32_t ecol = ecol_p + rep * ne;
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
#pragma unroll
                for (int k = 0; k < WP; ++k) tile[(size_t(cone) * WP + k) * ne + e] = out[k];
            }
            }
            if (mine && e == 0) {
                lmeta[cone] = (1u << WP) - 1u;                     // all sent, no failed bit
                folded[cone] = 1u;
            }
        }

        // ---- the inputs of the rows above, all levels at once: item q = (row in the order deepest level first, value
        // index of the block).  Requested here and not earlier: during the walk its registers are all in use; what the
        // items need is worked out from a copy of the thread's number that does not exist before this point.
        uint32_t tid_b = tid;
        asm volatile("" : "+v"(tid_b) : : "memory");
        const uint32_t NQ = (ncones - 1u) * ne;
        uint32_t jx = kNoRank, kx = 0;
        if (root != 0) {                              // the process that carries the root's number is process 0
            jx = fdiv(root - 1u, g.divW);
            kx = root - 1u - jx * g.W;
        }
        T xs[kFusedItems][WP];
        uint32_t ij[kFusedItems], ie[kFusedItems], il[kFusedItems], ip[kFusedItems];
#pragma unroll
        for (int i = 0; i < kFusedItems; ++i) {
            const uint32_t q = tid_b + uint32_t(i) * nthr;
            const bool valid = q < NQ;
            const uint32_t r = fdiv(valid ? q : 0u, fl.div_ne);
            const uint32_t el = (valid ? q : 0u) - r * ne;
            const uint32_t ec = pass * ne + el < g.E ? pass * ne + el : 0u;     // past the last value index: any valid address
            const uint32_t t = ncones - 1u - r;           // 2^l <= t < 2^(l+1) on level l of the part
            const uint32_t l = ilog2(t);
            const uint32_t p = (2u << l) - 1u - t;        // position on its level of the part
            const uint32_t j = (1u << (l + fl.dp)) - 1u + (part << l) + p;
            ij[i] = j; ie[i] = el; ip[i] = p;
            il[i] = (valid && pass * ne + el < g.E) ? l : kNoRank;
            const T* src = reinterpret_cast<const T*>(pay) + (size_t(1u + j * g.W)) * g.E + ec;
#pragma unroll
            for (int k = 0; k < WP; ++k) xs[i][k] = src[size_t(k) * g.E];
            if (j == jx) {
                const T x0 = reinterpret_cast<const T*>(pay)[ec];
#pragma unroll
                for (int k = 0; k < WP; ++k) xs[i][k] = kx == uint32_t(k) ? x0 : xs[i][k];
            }
        }
        __syncthreads();                                  // every wavefront has left its top rows

        // ---- the subtrees folded by the list kernel (an earlier launch): their top rows and words from the scratch area
        for (uint32_t c = wid; c < ncones; c += (nthr >> 6)) {
            if (top0 + cone0 + c < g.M && !folded[c]) {
                const T* src = reinterpret_cast<const T*>(wsS + td.out_off + size_t(cone0 + c) * g.RB);
                for (uint32_t i = lane; i < REl; i += 64u) {
                    const uint32_t k = fdiv(i, fl.div_ne), el = i - k * ne;
                    if (pass * ne + el < g.E) tile[size_t(c) * REl + i] = src[size_t(k) * g.E + pass * ne + el];
                }
                if (lane == 0) lmeta[c] = reinterpret_cast<const uint32_t*>(wsS + td.out_meta_off)[cone0 + c];
            }
        }
        __syncthreads();

        // ---- the levels above the deepest tier, out of LDS
        bool check_fail = false;
        if (ft.listed != 0)
            for (uint32_t q = 0; q < ft.n; ++q)
                if (ft.row[q] != kNoRank && ilog2(ft.row[q] + 1u) < td.dlo) check_fail = true;
        uint32_t im[kFusedItems];
        for (int l = int(dlo) - 1; l >= 0; --l) {
#pragma unroll
            for (int i = 0; i < kFusedItems; ++i) {
                if (il[i] == uint32_t(l)) {
                    const T* c0 = tile + size_t(2u * ip[i]) * REl + ie[i];
                    im[i] = fused_item<T, OP, WP>(ft, check_fail, ij[i], xs[i], c0, c0 + REl, ne, lmeta[2u * ip[i]],
                                                  lmeta[2u * ip[i] + 1u], pass == 0 && ie[i] == 0, uc_cnt, tree_cnt);
                }
            }
            __syncthreads();                              // the level below has been read
#pragma unroll
            for (int i = 0; i < kFusedItems; ++i) {
                if (il[i] == uint32_t(l)) {
                    T* dst = tile + size_t(ip[i]) * REl + ie[i];
#pragma unroll
                    for (int k = 0; k < WP; ++k) dst[size_t(k) * ne] = xs[i][k];
                    if (ie[i] == 0) lmeta[ip[i]] = im[i];
                }
            }
            __syncthreads();
        }
        if (fl.dp != 0u) {
            // ---- the part's top row goes on to the tiers above: messages [member][value index], sent and failed bits
            T* dst = reinterpret_cast<T*>(wsS + A.lift_off) + size_t(part) * g.W * g.E;
            for (uint32_t i = tid; i < REl; i += nthr) {
                const uint32_t k = fdiv(i, fl.div_ne), el = i - k * ne;
                if (pass * ne + el < g.E) dst[size_t(k) * g.E + pass * ne + el] = tile[i];
            }
            if (tid == 0 && pass == 0) reinterpret_cast<uint32_t*>(wsS + A.lift_meta_off)[part] = lmeta[0];
        } else if (!discard) {
        // ---- Algorithm "reduce at the root": lowest-numbered child whose message is present and reports no failure;
        // the root adds its own value iff that subtree holds no member of the root's group (children a .. f+1)
        const uint32_t cm = lmeta[0];
        const uint32_t okm = cm & ~(cm >> 16) & ((1u << WP) - 1u);
        st = kStOk;
        if (!ft.root_alive) st = kStRootFailed;
        else if (okm == 0) st = kStNoCleanSubtree;
        T* res = reinterpret_cast<T*>(A.result) + size_t(s) * g.E;
        const T* vroot = reinterpret_cast<const T*>(wsS + A.vroot_off);       // left by the list kernel (short last group)
        for (uint32_t el = tid; el < ne; el += nthr) {
            const uint32_t ec = pass * ne + el;
            if (ec >= g.E) continue;
            T val = T(0);
            if (st == kStOk) {
                const uint32_t ks = uint32_t(__ffs(int(okm))) - 1u;
                val = tile[size_t(ks) * ne + el];
                if (ks + 1u >= g.a) {
                    const T vr = g.a == 1 ? reinterpret_cast<const T*>(pay + size_t(root) * g.EB)[ec] : vroot[ec];
                    val = comb<T, OP>(vr, val);
                }
            }
            res[ec] = val;
        }
        }
    }

    // ---- message counters: one atomic per wavefront (the workgroup of the first block counts)
    if (A.msgs) {
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) {
            uc_cnt += __shfl_xor(uc_cnt, d);
            tree_cnt += __shfl_xor(tree_cnt, d);
        }
        if (lane == 0) {
            if (uc_cnt) atomicAdd(&A.msgs[size_t(s) * A.nmsg + 0], (unsigned long long)uc_cnt);
            if (tree_cnt) atomicAdd(&A.msgs[size_t(s) * A.nmsg + 1], (unsigned long long)tree_cnt);
        }
    }
    if (fl.dp == 0u && !discard && tid == 0 && pass == 0) A.status[s] = st;
}

#define FTRED_DECLARE_FUSED_LAUNCHER(NAME) \
    hipError_t launch_fused_##NAME(const RunArgs& A, const FusedLayout& fl, uint32_t grid, uint32_t lds, hipStream_t st);

FTRED_DECLARE_FUSED_LAUNCHER(i64_sum)
FTRED_DECLARE_FUSED_LAUNCHER(i64_bor)
FTRED_DECLARE_FUSED_LAUNCHER(u32_sum)
FTRED_DECLARE_FUSED_LAUNCHER(u32_bor)
FTRED_DECLARE_FUSED_LAUNCHER(f64_sum)

#define FTRED_DEFINE_FUSED_LAUNCHER(NAME, T, OP)                                                     \
    template <int WP>                                                                                \
    static hipError_t fused_wp_##NAME(const RunArgs& A, const FusedLayout& fl, uint32_t grid, uint32_t lds, hipStream_t st) \
    {                                                                                                \
        if (lds > 48u * 1024u) {      /* more dynamic LDS than a launch gets without asking */               \
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&fused_tree_kernel<T, OP, WP>),   \
                                               hipFuncAttributeMaxDynamicSharedMemorySize, int(lds));         \
            if (e != hipSuccess) return e;                                                           \
        }                                                                                            \
        hipLaunchKernelGGL((fused_tree_kernel<T, OP, WP>), dim3(grid), dim3(64u << fl.wshift), lds, st, A, fl); \
        return hipGetLastError();                                                                    \
    }                                                                                                \
    hipError_t launch_fused_##NAME(const RunArgs& A, const FusedLayout& fl, uint32_t grid, uint32_t lds, hipStream_t st) \
    {                                                                                                \
        FTRED_WAVE_WIDTH_SWITCH(A.g.W, fused_wp_##NAME, A, fl, grid, lds, st)                       \
    }

}  // namespace ftred

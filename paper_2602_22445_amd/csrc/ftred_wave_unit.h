// Deepest tier of the tree phase for one value per process (E == 1): eight LANES
// share one subtree of rows.
//
// With one value per process a row (= one up-correction group) is only W
// consecutive values.  A lane per subtree, as in the kernel for wider payloads, then
// reads 64 short pieces that lie 16 rows apart with every load, and the memory
// system delivers half of what it can.  Here the 64 lanes of a wavefront are eight
// sibling subtrees of height 4 times eight lanes, and the rows of every level of
// the eight subtrees are one contiguous run that the lanes read side by side:
//
//   lane q = 0..7 of a subtree reads rows 2q and 2q+1 of the subtree's level 4
//   (2W consecutive values), row q of level 3, and one row of the levels above:
//   lanes 0..3 the rows of level 2, lanes 4 and 5 the rows of level 1, lane 6 the
//   top; lane 7 has none.
//
// Each lane forms the up-correction values of its rows in the order of the rounds
// (Algorithm "Up-correction") and adds the tree messages of the level-4 rows to its
// level-3 row in registers (Algorithm "reduce at non-roots": the lower-numbered
// child first).  The three levels above take the messages of their children rows
// from the lanes that hold them, by lane permutation: the children of the row of
// lane q live in lanes 2q mod 8 and 2q mod 8 + 1 on every one of the three levels.
//
// The kernel runs the same subtrees as the kernel for wider payloads (every row
// exists, nobody listed as failed, no short last group); the relabelled rank (a
// root other than process 0) is patched into the row it belongs to.  The others are
// listed and run by the list kernels.  Output format as there.
//
// The wavefront does not stop at the top rows of its subtrees (UnitLayout::lift): the
// sibling subtrees of a group have one ancestor log2(subtrees per group) levels up,
// and the rows in between (seven per group of eight) are folded out of LDS by a lane
// each, with the per-row code of the kernel that folds a whole scenario (fused_item:
// up-correction in round order, the children's messages with their sent and failed
// bits).  The top rows of the listed subtrees are then needed here, so on this path the
// list kernels run in an earlier launch and leave them in the scratch area; one row
// per group goes on to the tier above, which starts that many levels higher.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ftred_fused.h"
#include "ftred_geom.h"
#include "ftred_kernels.h"
#include "ftred_wave.h"

namespace ftred {

constexpr uint32_t kUnitShift = 3;   // eight lanes per subtree, so eight subtrees per wavefront (fewer if the tier has fewer)

struct UnitLayout {
    uint32_t slot_shift;             // 2^slot_shift sibling subtrees per wavefront pass (<= 3)
    uint32_t group_shift;            // a wavefront walks through 2^group_shift such groups
    uint32_t lift;                   // levels above the subtrees' top rows that the wavefront folds as well (<= slot_shift)
};

// levels the kernel can fold above the top rows of its subtrees: the sibling subtrees of a group have one ancestor
// slot_shift levels up; the tier above must keep at least the root's children
inline uint32_t unit_lift(uint32_t dlo)
{
    const uint32_t sh = dlo < kUnitShift ? dlo : kUnitShift;
    return dlo == 0 ? 0u : (sh < dlo - 1u ? sh : dlo - 1u);
}

static_assert(kWaveH == 4, "the lane mapping below is written out for subtrees of height 4");

inline UnitLayout make_unit_layout(uint32_t dlo, uint32_t W)
{
    UnitLayout u;
    u.slot_shift = dlo < kUnitShift ? dlo : kUnitShift;
    // Two groups per wavefront measured fastest for rows of 72 bytes (one: 3 % slower, eight: as slow as one), and
    // within 3 % of the best for every other width but the powers of two: rows of 16, 32, 64 or 128 bytes put the
    // groups of a wavefront, a power of two of rows apart, onto the same channels, and eight groups per wavefront
    // are 12 to 27 % faster there (W = 8, P = 16384: 1.17 against 1.60 ms per 4 GiB; W = 4: 0.92 against 1.12).
    // The plan's flags can ask for another number.
    const uint32_t most = dlo - u.slot_shift;
    const uint32_t want = (W & (W - 1u)) == 0u ? 3u : 1u;
    u.group_shift = want < most ? want : most;
    u.lift = 0;
    return u;
}

template <class T, int OP, int WP>
struct UnitRow {
    // the W inputs of row j as they lie in memory
    static __device__ __forceinline__ void load(const T* x, uint32_t j, T (&r)[WP])
    {
        const T* p = x + 1u + size_t(j) * uint32_t(WP);
#pragma unroll
        for (int k = 0; k < WP; ++k) r[k] = p[k];
    }
    // the process that carries the root's number (member kx of row jx) holds x0
    static __device__ __forceinline__ void patch(uint32_t j, uint32_t jx, uint32_t kx, T x0, T (&r)[WP])
    {
        const bool here = j == jx;
#pragma unroll
        for (int k = 0; k < WP; ++k) r[k] = (here && kx == uint32_t(k)) ? x0 : r[k];
    }
    // up-correction: in round t member i receives the input of member (i - t) mod W
    static __device__ __forceinline__ void correct(const T (&r)[WP], T (&v)[WP])
    {
#pragma unroll
        for (int i = 0; i < WP; ++i) {
            T acc = r[i];
#pragma unroll
            for (int t = 1; t < WP; ++t) acc = comb<T, OP>(acc, r[exchange_source(uint32_t(i), uint32_t(t), uint32_t(WP))]);
            v[i] = acc;
        }
    }
};

// what a lane reads for one group of subtrees
template <class T, int WP>
struct UnitRows {
    T ra[WP], rb[WP], rc[WP], ru[WP];      // rows 2q, 2q+1 of level 4, row q of level 3, the lane's row above
};

template <class T, int OP, int WP>
__global__ void __launch_bounds__(kWaveThreads) unit_tier_kernel(RunArgs A, UnitLayout ul)
{
    const Geom& g = A.g;
    const TierDesc& td = A.tiers[0];
    const uint32_t lane = threadIdx.x;
    const uint32_t wshift = td.dlo - ul.slot_shift - ul.group_shift;   // wavefronts per scenario = 2^wshift
    const uint32_t sv = blockIdx.x >> wshift;                  // scenario, or S + retry entry
    const uint32_t top0 = (1u << td.dlo) - 1u;
    // The groups of a wavefront lie 2^wshift groups apart: the wavefronts that run side by side then read rows
    // that lie side by side whichever of its groups each of them has reached.
    const uint32_t wid = blockIdx.x & ((1u << wshift) - 1u);
    auto group_at = [&](uint32_t gi) { return wid + (gi << wshift); };
    if (top0 + (wid << ul.slot_shift) >= g.M) return;          // no such rows

    const uint32_t slot = lane >> 3, q = lane & 7u;
    const bool active = slot < (1u << ul.slot_shift);
    // the lane's row above level 3, as an index into the subtree (top 0, children 2i+1, 2i+2)
    const uint32_t ui = q < 4u ? 3u + q : (q < 6u ? q - 3u : 0u);
    const uint32_t ulev = q < 4u ? 2u : (q < 6u ? 1u : 0u);
    const uint32_t src = (lane & ~7u) | ((2u * q) & 7u);       // lane of the lower-numbered child row, levels 2..0

    // the payload does not depend on the failures: the first rows are requested before anything else is read
    uint32_t s = sv;
    if (sv >= A.S) {
        const uint32_t kk = sv - A.S;
        if (kk >= *A.retry_count) return;
        s = __builtin_amdgcn_readfirstlane(A.retry_list[2u * kk]);
    }
    const T* x = reinterpret_cast<const T*>(A.payload + size_t(s) * A.scen_stride_bytes);
    const uint32_t nfull = g.a > 1u ? g.M - 1u : g.M;          // rows whose W inputs all lie in memory
    const uint32_t ngroups = 1u << ul.group_shift;
    using Row = UnitRow<T, OP, WP>;

    // the lane's rows in the subtree below row rs
    auto row4 = [&](uint32_t rs) { return ((rs + 1u) << 4) - 1u + 2u * q; };
    auto row3 = [&](uint32_t rs) { return ((rs + 1u) << 3) - 1u + q; };
    auto rowu = [&](uint32_t rs) { return ((rs + 1u) << ulev) - 1u + (ui - ((1u << ulev) - 1u)); };
    // requests the rows of group gi that exist, whoever folds that subtree in the end
    auto request = [&](uint32_t gi, UnitRows<T, WP>& R) {
        const uint32_t rs = top0 + (group_at(gi) << ul.slot_shift) + (active ? slot : 0u);
#pragma unroll
        for (int k = 0; k < WP; ++k) R.ra[k] = R.rb[k] = R.rc[k] = R.ru[k] = T(0);
        if (!active) return;
        if (row4(rs) + 1u < nfull) {
            Row::load(x, row4(rs), R.ra);
            Row::load(x, row4(rs) + 1u, R.rb);
        }
        if (row3(rs) < nfull) Row::load(x, row3(rs), R.rc);
        if (q < 7u && rowu(rs) < nfull) Row::load(x, rowu(rs), R.ru);
    };
    // the lane's entry of the failure list, for the subtrees that are not folded here
    const uint32_t F = g.f > 0 ? g.f : 1;
    const uint32_t listed = lane < g.f ? A.fail_rank[size_t(s) * F + lane] : kNoRank;
    // the whole entry, for the levels above the subtrees: requested here, used after the walk
    FailRaw fraw;
    fraw.rank = kNoRank; fraw.round = 0;
    if (ul.lift != 0u) fraw = failtab_load(g, A.fail_rank, A.fail_round, s);
    UnitRows<T, WP> R;
    request(0, R);

    uint32_t root = 0, status = kStOk;
    unsigned char* wsS;
    if (sv < A.S) {
        status = A.status[s];
        if (A.attempts) root = A.attempts[s];                  // roots tried; the last one is alive
        else if (A.root) root = A.root[s];
        if (A.attempts) root = root > 0 ? root - 1u : 0u;
        wsS = A.ws + size_t(s) * A.ws_stride;
    } else {
        const uint32_t kk = sv - A.S;
        root = A.retry_list[2u * kk + 1u];
        wsS = A.retry_ws + size_t(kk) * A.ws_stride;
    }
    status = __builtin_amdgcn_readfirstlane(status);
    root = __builtin_amdgcn_readfirstlane(root);
    if (status == kStBadFailureSet) return;
    // the subtrees that go to the list kernels, one per lane (at most f + 1 of them, f + 1 <= 64)
    const uint32_t special = subtree_of_row(special_row_of_lane(g, td.dlo, listed, root, lane), td.dlo);
    // section "Reduce": the root swaps numbers with process 0
    uint32_t jx = kNoRank, kx = 0;
    T x0 = T(0);
    if (root != 0) {
        jx = fdiv(root - 1u, g.divW);
        kx = root - 1u - jx * g.W;
        x0 = x[0];
    }
    // the top rows wait in LDS for one run of stores at the end: a store between the requests would make every
    // wait for rows a wait for that store as well
    extern __shared__ __align__(16) unsigned char unit_lds[];
    FailTab& ft = *reinterpret_cast<FailTab*>(unit_lds);                        // used by the levels above only
    T* tops = reinterpret_cast<T*>(unit_lds + sizeof(FailTab));                // [groups][slots][W]
    uint32_t* folded = reinterpret_cast<uint32_t*>(tops + (size_t(WP) << (ul.group_shift + ul.slot_shift)));

    // The levels above (ul.lift of them): the 2^slot_shift sibling subtrees of a group have a common ancestor
    // slot_shift levels up; lane 8 gi + r takes row r of group gi's part of the tree in heap order (0 = that
    // ancestor, children 2r + 1 and 2r + 2, the top rows of the subtrees below the last level).  Its inputs are
    // requested here, ahead of the walk.
    const uint32_t nc = 1u << ul.slot_shift;
    const uint32_t ur = lane & 7u, ugi = lane >> 3;
    const uint32_t uh = ul.slot_shift - ilog2(ur + 1u);        // height above the top rows (only for ur < nc - 1)
    const bool lifts = ul.lift != 0u && ugi < ngroups && ur + 1u < nc && uh <= ul.lift;
    uint32_t uj = 0;
    T ux[WP];
#pragma unroll
    for (int k = 0; k < WP; ++k) ux[k] = T(0);
    if (lifts) {
        const uint32_t c0 = group_at(ugi) << ul.slot_shift;   // first subtree of the group
        const uint32_t pos = (c0 >> uh) + (ur + 1u - (nc >> uh));
        uj = (1u << (td.dlo - uh)) - 1u + pos;
        Row::load(x, uj, ux);
    }

    for (uint32_t gi = 0; gi < ngroups; ++gi) {
        UnitRows<T, WP> C = R;
        if (gi + 1u < ngroups) request(gi + 1u, R);            // in flight while this group is folded

        const uint32_t cone = (group_at(gi) << ul.slot_shift) + (active ? slot : 0u);
        const uint32_t rs = top0 + cone;                       // top row of the lane's subtree
        // shape of the subtree: complete with or without the bottom level (a ragged one is listed)
        const uint32_t last_leaf = ((rs + 2u) << kWaveH) - 2u;
        const bool bottom = last_leaf < g.M;
        bool handover = false;
        const uint32_t cone_w = group_at(gi) << ul.slot_shift;
        unsigned long long hits = __ballot(special - cone_w < (1u << ul.slot_shift));    // rarely any
        while (hits != 0ull) {
            const int e = __ffsll(hits) - 1;
            hits &= hits - 1ull;
            if (uint32_t(__builtin_amdgcn_readlane(int(special), e)) == cone) handover = true;
        }
        const bool mine = active && rs < g.M && !handover;
        Row::patch(row4(rs), jx, kx, x0, C.ra);
        Row::patch(row4(rs) + 1u, jx, kx, x0, C.rb);
        Row::patch(row3(rs), jx, kx, x0, C.rc);
        Row::patch(q < 7u ? rowu(rs) : kNoRank - 1u, jx, kx, x0, C.ru);

        T va[WP], vb[WP], m[WP], vu[WP];
        Row::correct(C.ra, va);
        Row::correct(C.rb, vb);
        Row::correct(C.rc, m);
        Row::correct(C.ru, vu);
        // level 3: the two rows of level 4 are this lane's own
#pragma unroll
        for (int k = 0; k < WP; ++k) m[k] = bottom ? comb<T, OP>(comb<T, OP>(m[k], va[k]), vb[k]) : m[k];
        // levels 2, 1, 0: the children rows' messages come from lanes src and src + 1; all lanes take part in the
        // permutation, the lanes of the level keep the result
#pragma unroll
        for (int lev = 2; lev >= 0; --lev) {
            const bool at = ulev == uint32_t(lev) && q < 7u;
#pragma unroll
            for (int k = 0; k < WP; ++k) {
                const T lo = __shfl(m[k], int(src));
                const T hi = __shfl(m[k], int(src + 1u));
                m[k] = at ? comb<T, OP>(comb<T, OP>(vu[k], lo), hi) : m[k];
            }
        }
        // lane 6 holds the top row
        if (active && q == 6u) {
            const uint32_t at = (gi << ul.slot_shift) + slot;
#pragma unroll
            for (int k = 0; k < WP; ++k) tops[at * uint32_t(WP) + k] = m[k];
            folded[at] = mine ? 1u : 0u;
        }
    }
    __syncthreads();
    const uint32_t ncones = ngroups << ul.slot_shift, smask = (1u << ul.slot_shift) - 1u;
    auto cone_of = [&](uint32_t c) { return (group_at(c >> ul.slot_shift) << ul.slot_shift) + (c & smask); };
    if (ul.lift != 0u) {
        // ---- the levels above the subtrees, out of LDS (as in the kernel that folds a whole scenario)
        uint32_t* lmeta = folded + ncones;                                         // sent / failed bits of the top rows
        T* up = reinterpret_cast<T*>(lmeta + ncones);                              // [groups][nc - 1 rows][W]; 2 ncones words before it
        uint32_t* upmeta = reinterpret_cast<uint32_t*>(up + size_t(ngroups) * (nc - 1u) * uint32_t(WP));
        uint32_t base = 0;
        if (sv >= A.S || A.attempts) base = root * g.Ratt;     // rounds of the attempt (allreduce)
        failtab_store(ft, g, failtab_compute(g, fraw, root, base));
        // the top rows of the subtrees the list kernels folded (an earlier launch) come in from the scratch area
        for (uint32_t c = lane; c < ncones; c += kWaveThreads) {
            if (folded[c]) {
                lmeta[c] = (1u << WP) - 1u;                    // all sent, no failed bit
            } else {
                const T* src = reinterpret_cast<const T*>(wsS + td.out_off) + size_t(cone_of(c)) * uint32_t(WP);
#pragma unroll
                for (int k = 0; k < WP; ++k) tops[c * uint32_t(WP) + k] = src[k];
                lmeta[c] = reinterpret_cast<const uint32_t*>(wsS + td.out_meta_off)[cone_of(c)];
            }
        }
        __syncthreads();
        bool check_fail = false, row_listed = false;
        if (ft.listed != 0)
            for (uint32_t qq = 0; qq < ft.n; ++qq) {
                if (ft.row[qq] == kNoRank) continue;
                const uint32_t d = ilog2(ft.row[qq] + 1u);
                if (d + ul.lift >= td.dlo && d < td.dlo) check_fail = true;
                if (lifts && ft.row[qq] == uj) row_listed = true;
            }
        Row::patch(lifts ? uj : kNoRank - 1u, jx, kx, x0, ux);
        uint32_t uc_cnt = 0, tree_cnt = 0;
        for (uint32_t h = 1; h <= ul.lift; ++h) {
            if (lifts && uh == h) {
                // children: rows 2 ur + 1, 2 ur + 2 of the group's part; below the last level the top rows
                const uint32_t ci = 2u * ur + 1u;
                const T* c0p;
                uint32_t cm0, cm1;
                if (ci >= nc - 1u) {
                    const uint32_t at = (ugi << ul.slot_shift) + (ci - (nc - 1u));
                    c0p = tops + size_t(at) * uint32_t(WP);
                    cm0 = lmeta[at]; cm1 = lmeta[at + 1u];
                } else {
                    c0p = up + (size_t(ugi) * (nc - 1u) + ci) * uint32_t(WP);
                    cm0 = upmeta[ugi * (nc - 1u) + ci]; cm1 = upmeta[ugi * (nc - 1u) + ci + 1u];
                }
                const uint32_t mw = fused_item<T, OP, WP>(ft, check_fail, uj, ux, c0p, c0p + WP, 1u, cm0, cm1, row_listed,
                                                          uc_cnt, tree_cnt);
                T* dst = up + (size_t(ugi) * (nc - 1u) + ur) * uint32_t(WP);
#pragma unroll
                for (int k = 0; k < WP; ++k) dst[k] = ux[k];
                upmeta[ugi * (nc - 1u) + ur] = mw;
                if (h == ul.lift) {
                    // the rows the tier above takes as its children
                    const uint32_t pos = uj + 1u - (1u << (td.dlo - h));
                    T* out = reinterpret_cast<T*>(wsS + A.lift_off) + size_t(pos) * uint32_t(WP);
#pragma unroll
                    for (int k = 0; k < WP; ++k) out[k] = ux[k];
                    reinterpret_cast<uint32_t*>(wsS + A.lift_meta_off)[pos] = mw;
                }
            }
            __syncthreads();
        }
        // rows with listed members are counted message by message (the others by their number, beforehand)
        if (A.msgs && __ballot(uc_cnt | tree_cnt) != 0ull) {
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
        return;
    }
    // the top rows go to the tier above: the subtrees of a group are neighbours, so are their rows there
    T* dst = reinterpret_cast<T*>(wsS + td.out_off);
    for (uint32_t i = lane; i < ncones * uint32_t(WP); i += kWaveThreads) {
        const uint32_t c = i / uint32_t(WP), k = i - c * uint32_t(WP);
        if (folded[c]) dst[size_t(cone_of(c)) * uint32_t(WP) + k] = tops[i];
    }
    for (uint32_t c = lane; c < ncones; c += kWaveThreads)
        if (folded[c]) reinterpret_cast<uint32_t*>(wsS + td.out_meta_off)[cone_of(c)] = (1u << g.W) - 1u;   // all sent, no failed bit
    if (A.info) {                     // and nobody in these subtrees missed a message: empty lists
        uint16_t* mk = reinterpret_cast<uint16_t*>(wsS + td.out_mask_off);
        for (uint32_t i = lane; i < ncones * uint32_t(WP); i += kWaveThreads) {
            const uint32_t c = i / uint32_t(WP), k = i - c * uint32_t(WP);
            if (folded[c]) mk[size_t(cone_of(c)) * uint32_t(WP) + k] = 0;
        }
    }
}

// LDS of one wavefront of the kernel above
template <class T>
inline uint32_t unit_lds_bytes(const UnitLayout& ul, uint32_t W)
{
    const uint32_t cones = 1u << (ul.group_shift + ul.slot_shift), groups = 1u << ul.group_shift;
    uint32_t n = uint32_t(sizeof(FailTab)) + cones * W * uint32_t(sizeof(T)) + cones * 4u;
    if (ul.lift) {
        // words of the top rows, the rows above them and their words
        const uint32_t rows = groups * ((1u << ul.slot_shift) - 1u);
        n += cones * 4u + rows * W * uint32_t(sizeof(T)) + rows * 4u;
    }
    return n;
}

#define FTRED_DECLARE_UNIT_LAUNCHER(NAME) \
    hipError_t launch_unit_##NAME(const RunArgs& A, const UnitLayout& ul, uint32_t grid, hipStream_t st);

FTRED_DECLARE_UNIT_LAUNCHER(i64_sum)
FTRED_DECLARE_UNIT_LAUNCHER(i64_bor)
FTRED_DECLARE_UNIT_LAUNCHER(u32_sum)
FTRED_DECLARE_UNIT_LAUNCHER(u32_bor)
FTRED_DECLARE_UNIT_LAUNCHER(f64_sum)

#define FTRED_DEFINE_UNIT_LAUNCHER(NAME, T, OP)                                                     \
    template <int WP>                                                                               \
    static hipError_t unit_wp_##NAME(const RunArgs& A, const UnitLayout& ul, uint32_t grid, hipStream_t st) \
    {                                                                                               \
        hipLaunchKernelGGL((unit_tier_kernel<T, OP, WP>), dim3(grid), dim3(kWaveThreads),           \
                           unit_lds_bytes<T>(ul, uint32_t(WP)), st, A, ul);                         \
        return hipGetLastError();                                                                   \
    }                                                                                               \
    hipError_t launch_unit_##NAME(const RunArgs& A, const UnitLayout& ul, uint32_t grid, hipStream_t st) \
    {                                                                                               \
        if (A.g.E != 1u) return hipErrorInvalidValue;                                               \
        FTRED_WAVE_WIDTH_SWITCH_WIDE(A.g.W, unit_wp_##NAME, A, ul, grid, st)                        \
    }

}  // namespace ftred

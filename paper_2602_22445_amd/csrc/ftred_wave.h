// Deepest tier of the tree phase, one wavefront per subtree of rows.
//
// A row (= one up-correction group = the j-th process of each subtree of the
// root) is W*E values that are consecutive in HBM.  Here a LANE owns a COLUMN
// (member k, value index e) of the rows it visits:
//   - the input of row j is one coalesced load: lane (k, e) reads value e of
//     member k, the lanes of a row read consecutive addresses;
//   - up-correction (Algorithm "Up-correction") needs the other members' inputs of
//     the same row and value index: the wavefront writes the row to a small LDS
//     exchange buffer and lane (k, e) reads members k-1, k-2, .. (mod group size)
//     in the order of the rounds;
//   - the tree phase (Algorithm "reduce at non-roots") needs the messages of the
//     two children rows, which are the SAME lane's earlier results: registers.
// A wavefront owns the rows of a subtree of height H below one row of depth dlo
// (31 rows for H = 4), loads all of them first (everything in flight at once) and
// folds them bottom-up.  No workgroup barrier, no staging pass, no index
// arithmetic per element.  If W*E < 64, several sibling subtrees sit side by side
// in the lanes ("slots"); if W*E > 64 the value indices are walked in passes.
//
// This kernel runs the subtrees in which every row exists, nothing is listed as
// failed, and neither the relabelled ranks nor the short last group occur (fully
// unrolled, unmasked code).  The few others (at most f + 3 wavefronts per
// scenario) are appended to a list and run by the general LDS-tile kernel, which
// carries per-member liveness, sent and failed bits (section "Failure
// information": the single failed bit).
//
// The subtree's top row leaves through the scratch area in the format the upper
// tiers read: W*E values and one word (bits 0..15 sent, 16..31 failed bit).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ftred_geom.h"
#include "ftred_kernels.h"

namespace ftred {

constexpr int kWaveH = 4;            // height of the subtree one wavefront owns
constexpr int kWaveNBuf = 2;         // exchange buffers per wavefront (two sibling rows per step)
constexpr int kWavesPerWg = kThreads / 64;

struct WaveLayout {                  // how the 64 lanes map to (slot, member, value index)
    uint32_t ne;                     // value indices per pass
    uint32_t slot_shift;             // 2^slot_shift sibling subtrees per wavefront
    uint32_t nact;                   // active lanes = slots * W * ne
    uint32_t passes;                 // ceil(E / ne)
};

inline WaveLayout make_wave_layout(const Geom& g, uint32_t dlo)
{
    WaveLayout w;
    w.ne = g.E < 64u / g.W ? g.E : 64u / g.W;
    uint32_t slots = 64u / (g.W * w.ne), sh = 0;
    while ((2u << sh) <= slots && sh < dlo) ++sh;
    w.slot_shift = sh;
    w.nact = (1u << sh) * g.W * w.ne;
    w.passes = (g.E + w.ne - 1u) / w.ne;
    return w;
}

struct WaveLds {                     // per wavefront
    unsigned long long exch[kWaveNBuf][64];      // rows in exchange between the lanes of a group
};

template <class T>
__device__ __forceinline__ unsigned long long to_bits(T v)
{
    if constexpr (sizeof(T) == 8) return __builtin_bit_cast(unsigned long long, v);
    else return (unsigned long long)__builtin_bit_cast(uint32_t, v);
}
template <class T>
__device__ __forceinline__ T from_bits(unsigned long long b)
{
    if constexpr (sizeof(T) == 8) return __builtin_bit_cast(T, b);
    else return __builtin_bit_cast(T, uint32_t(b));
}

constexpr int cx_ilog2(int x) { return x <= 1 ? 0 : 1 + cx_ilog2(x / 2); }

// ---- PURE path: every row exists, every member is alive, groups have W members.
// EXACT: W == WP at compile time (straight-line code); otherwise WP >= W and the
// surplus rounds are computed and dropped by a select (no branch).
template <class T, int OP, int WP, bool EXACT, int HH>
__device__ __forceinline__ T pure_subtree(const Geom& g, const unsigned char* pay, uint32_t r0,
                                          const uint32_t (&laneoff)[kWaveH + 1], unsigned char* eb,
                                          const uint32_t (&rd_off)[WP] /* byte offsets of members k-t */)
{
    constexpr int NR = (2 << HH) - 1;
    T x[NR];
    // all rows in flight at once
#pragma unroll
    for (int li = 0; li < NR; ++li) {
        const int l = cx_ilog2(li + 1);
        const uint32_t i = uint32_t(li) - ((1u << l) - 1u);
        const uint32_t j0 = ((r0 + 1u) << l) - 1u + i;                 // row of slot 0 (wave-uniform)
        const uint32_t off = (1u + j0 * g.W) * g.EB + laneoff[l];      // wave-uniform row + lane offset
        x[li] = *reinterpret_cast<const T*>(pay + off);                 // scalar base + 32-bit offset
    }
    // bottom-up over the heap order (children have larger indices than parents), two
    // sibling rows per step: both rows are exchanged through LDS together, so one
    // LDS round trip serves two rows.  The compiler barriers keep the steps apart
    // (without them every LDS read is hoisted to the front and the registers run
    // out).
    auto fold = [&](const T (&y)[WP], T acc) -> T {
#pragma unroll
        for (int t = 1; t < WP; ++t) {
            const T r = comb<T, OP>(acc, y[t]);
            if constexpr (EXACT) acc = r; else acc = uint32_t(t) < g.W ? r : acc;
        }
        return acc;
    };
#pragma unroll
    for (int li = NR - 1; li >= 1; li -= 2) {          // rows li-1 (left) and li (right) are siblings
        unsigned char* bufa = eb;
        unsigned char* bufb = eb + 64 * 8;
        *reinterpret_cast<T*>(bufa + rd_off[0]) = x[li - 1];
        *reinterpret_cast<T*>(bufb + rd_off[0]) = x[li];
        __builtin_amdgcn_wave_barrier();          // both rows are written before any lane reads them
        T ya[WP], yb[WP];
#pragma unroll
        for (int t = 1; t < WP; ++t) {
            ya[t] = *reinterpret_cast<const T*>(bufa + rd_off[t]);
            yb[t] = *reinterpret_cast<const T*>(bufb + rd_off[t]);
        }
        T a = fold(ya, x[li - 1]);
        T b = fold(yb, x[li]);
        if (2 * li + 2 < NR) {
            a = comb<T, OP>(comb<T, OP>(a, x[2 * (li - 1) + 1]), x[2 * (li - 1) + 2]);
            b = comb<T, OP>(comb<T, OP>(b, x[2 * li + 1]), x[2 * li + 2]);
        }
        // the step's results are complete, and no LDS traffic of the next step starts, before this point
        asm volatile("" : "+v"(a), "+v"(b) : : "memory");
        x[li - 1] = a;
        x[li] = b;
    }
    {
        *reinterpret_cast<T*>(eb + rd_off[0]) = x[0];
        __builtin_amdgcn_wave_barrier();
        T y[WP];
#pragma unroll
        for (int t = 1; t < WP; ++t) y[t] = *reinterpret_cast<const T*>(eb + rd_off[t]);
        T a = fold(y, x[0]);
        if (NR > 1) a = comb<T, OP>(comb<T, OP>(a, x[1]), x[2]);
        x[0] = a;
    }
    return x[0];
}

template <class T, int OP, int WP, bool EXACT>
__global__ void __launch_bounds__(kThreads) wave_tier_kernel(RunArgs A, WaveLayout wl)
{
    __shared__ FailTab ft;
    __shared__ WaveLds wlds[kWavesPerWg];
    const Geom& g = A.g;
    const TierDesc& td = A.tiers[0];
    const uint32_t tid = threadIdx.x;
    const uint32_t lane = tid & 63u, wv = tid >> 6;
    // workgroup -> (scenario or retry entry, group of 4 wavefronts); wavefront -> 2^slot_shift subtrees
    const uint32_t wshift = td.dlo - wl.slot_shift;            // wavefronts per scenario = 2^wshift
    const uint32_t gshift = wshift >= 2 ? wshift - 2u : 0u;    // workgroups per scenario = 2^gshift
    const uint32_t sv = blockIdx.x >> gshift;
    const uint32_t wave_in_scen = ((blockIdx.x & ((1u << gshift) - 1u)) << 2) + wv;

    uint32_t s = sv, root = 0, base = 0;
    unsigned char* wsS;
    if (sv >= A.S) {
        const uint32_t kk = sv - A.S;
        if (kk >= *A.retry_count) return;
        s = __builtin_amdgcn_readfirstlane(A.retry_list[2u * kk]);
        root = A.retry_list[2u * kk + 1u];
        base = root * g.Ratt;
        wsS = A.retry_ws + size_t(kk) * A.ws_stride;
    } else {
        if (A.status[s] == kStBadFailureSet) return;
        if (A.attempts) {
            root = A.attempts[s] - 1u;
            base = root * g.Ratt;
        } else if (A.root) {
            root = A.root[s];
        }
        wsS = A.ws + size_t(s) * A.ws_stride;
    }
    // wave-uniform values loaded from memory: keep them in scalar registers
    s = __builtin_amdgcn_readfirstlane(s);
    root = __builtin_amdgcn_readfirstlane(root);
    base = __builtin_amdgcn_readfirstlane(base);
    load_failtab(ft, g, A.fail_rank, A.fail_round, s, root, base);
    __syncthreads();
    const unsigned char* pay = A.payload + size_t(s) * A.scen_stride_bytes;

    uint32_t uc_cnt = 0, tree_cnt = 0;
    const uint32_t top0 = (1u << td.dlo) - 1u;
    const uint32_t cone0 = wave_in_scen << wl.slot_shift;      // first subtree of this wavefront
    const uint32_t r0 = top0 + cone0;                          // its top row
    const bool wave_has_work = wave_in_scen < (1u << wshift) && r0 < g.M;
    if (wave_has_work && lane < wl.nact) {
        // lane -> (slot, member k, value index e)
        const uint32_t per_slot = g.W * wl.ne;
        const uint32_t slot = lane / per_slot;
        const uint32_t k = (lane - slot * per_slot) / wl.ne;
        const uint32_t e = lane - slot * per_slot - k * wl.ne;
        const uint32_t slot_lane0 = slot * per_slot;
        WaveLds& L = wlds[wv];

        // which path?  wave-uniform
        const uint32_t nslots = 1u << wl.slot_shift;
        const uint32_t rlast = r0 + nslots - 1u;                               // top row of the last slot
        const uint32_t first_leaf = ((r0 + 1u) << kWaveH) - 1u;                // first row of the bottom level
        const uint32_t last_leaf = ((rlast + 2u) << kWaveH) - 2u;              // last row of the bottom level
        const uint32_t last_leaf_m1 = ((rlast + 2u) << (kWaveH - 1)) - 2u;     // ... of the level above it
        bool checked = false;
        int pure_h = kWaveH;
        if (last_leaf < g.M) pure_h = kWaveH;
        else if (first_leaf >= g.M && last_leaf_m1 < g.M) pure_h = kWaveH - 1;
        else checked = true;
        // the short last group (root as a member), the relabelled ranks, listed processes
        {
            auto in_span = [&](uint32_t jr) -> bool {
                // is row jr inside one of this wavefront's subtrees?
                const uint32_t d = ilog2(jr + 1u);
                if (d < td.dlo || d > td.dlo + uint32_t(kWaveH)) return false;
                const uint32_t anc = ((jr + 1u) >> (d - td.dlo)) - 1u;
                return anc >= r0 && anc <= rlast;
            };
            if (g.a > 1 && in_span(g.M - 1u)) checked = true;
            if (root != 0 && in_span(fdiv(root - 1u, g.divW))) checked = true;
            if (ft.listed != 0)
                for (uint32_t q = 0; q < ft.n; ++q)
                    if (ft.row[q] != kNoRank && in_span(ft.row[q])) checked = true;
        }

        if (checked) {
            // not for this kernel: hand the subtrees to the general (LDS tile) kernel
            if (lane == 0) {
                const uint32_t n = atomicAdd(A.fix_count, 1u);
                A.fix_list[2u * n] = sv;
                A.fix_list[2u * n + 1u] = cone0;
            }
        }
        for (uint32_t pass = 0; pass < wl.passes && !checked; ++pass) {
            const uint32_t ecol = pass * wl.ne + e;
            if (ecol >= g.E) break;
            const uint32_t colbyte = (k * g.E + ecol) * g.esz;
            T out;
            {
                uint32_t laneoff[kWaveH + 1];
#pragma unroll
                for (int l = 0; l <= kWaveH; ++l) laneoff[l] = colbyte + slot * (g.RB << l);
                uint32_t rd_off[WP];
#pragma unroll
                for (int t = 0; t < WP; ++t) {
                    const uint32_t idx = (uint32_t(t) < g.W) ? (k >= uint32_t(t) ? k - uint32_t(t) : k + g.W - uint32_t(t)) : k;
                    rd_off[t] = (slot_lane0 + idx * wl.ne + e) * 8u;
                }
                unsigned char* eb = reinterpret_cast<unsigned char*>(&L.exch[0][0]);
                if (pure_h == kWaveH) out = pure_subtree<T, OP, WP, EXACT, kWaveH>(g, pay, r0, laneoff, eb, rd_off);
                else out = pure_subtree<T, OP, WP, EXACT, kWaveH - 1>(g, pay, r0, laneoff, eb, rd_off);
                if (pass == 0 && lane == 0) {
                    const uint32_t nrows = nslots * ((2u << pure_h) - 1u);
                    uc_cnt += nrows * g.W * (g.W - 1u);
                    tree_cnt += nrows * g.W;
                }
            }
            // the top row of the subtree goes to the tier above
            const uint32_t cone = cone0 + slot;
            if (top0 + cone < g.M) {
                *reinterpret_cast<T*>(wsS + td.out_off + size_t(cone) * g.RB + colbyte) = out;
                if (pass == 0 && e == 0) {
                    if (k == 0) reinterpret_cast<uint32_t*>(wsS + td.out_meta_off)[cone] = (1u << g.W) - 1u;
                }
            }
        }
    }
    if (A.msgs) {
        if (uc_cnt) atomicAdd(&ft.cnt_uc, uc_cnt);
        if (tree_cnt) atomicAdd(&ft.cnt_tree, tree_cnt);
        __syncthreads();
        if (tid == 0) {
            if (ft.cnt_uc) atomicAdd(&A.msgs[size_t(s) * A.nmsg + 0], (unsigned long long)ft.cnt_uc);
            if (ft.cnt_tree) atomicAdd(&A.msgs[size_t(s) * A.nmsg + 1], (unsigned long long)ft.cnt_tree);
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
    template <int WP, bool EXACT>                                                                   \
    static hipError_t wave_wp_##NAME(const RunArgs& A, const WaveLayout& wl, uint32_t grid, hipStream_t st) \
    {                                                                                               \
        hipLaunchKernelGGL((wave_tier_kernel<T, OP, WP, EXACT>), dim3(grid), dim3(kThreads), 0, st, A, wl); \
        return hipGetLastError();                                                                   \
    }                                                                                               \
    hipError_t launch_wave_##NAME(const RunArgs& A, const WaveLayout& wl, uint32_t grid, hipStream_t st) \
    {                                                                                               \
        switch (A.g.W) {          /* group widths with straight-line code; one generic kernel else */ \
            case 2: return wave_wp_##NAME<2, true>(A, wl, grid, st);                                \
            case 3: return wave_wp_##NAME<3, true>(A, wl, grid, st);                                \
            case 4: return wave_wp_##NAME<4, true>(A, wl, grid, st);                                \
            case 5: return wave_wp_##NAME<5, true>(A, wl, grid, st);                                \
            case 9: return wave_wp_##NAME<9, true>(A, wl, grid, st);                                \
            default: return wave_wp_##NAME<16, false>(A, wl, grid, st);                             \
        }                                                                                           \
    }

}  // namespace ftred

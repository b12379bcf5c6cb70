// Device code of the up-correction phase, the tree phase and the root's choice
// (Algorithms "Up-correction", "reduce at non-roots", "reduce at the root").
//
// Work decomposition.  A "row" j is one up-correction group = the j-th process
// of each of the W = f+1 subtrees of the root; its payload is W*E consecutive
// values in HBM.  Rows form a binary heap (children of row j: 2j+1, 2j+2), the
// same heap in every subtree, so the tree phase is a heap reduction over rows
// with W*E independent columns.  A workgroup owns a "cone": the rows below one
// row of depth dlo, down to depth dhi.  Rows of one depth inside a cone are
// consecutive in HBM, so the cone is staged into LDS with flat coalesced 16-byte
// loads, then reduced level by level (deepest first) out of LDS: each round's
// senders are the LDS-resident frontier of the level below.  Trees too tall for
// LDS are cut into tiers; a tier's top rows go through a small scratch area in
// HBM to the tier above.
//
// One thread handles one (row, value index) item: it reads the W inputs of the
// group, forms the W up-correction values in the fixed order of the rounds,
// adds what the two children rows sent, and writes the W tree messages back in
// place.  Liveness comes from the scenario's failure list (at most f entries),
// held in LDS.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "ftred_geom.h"

namespace ftred {

constexpr int kThreads = 256;
constexpr int kMaxTiers = 8;
constexpr int kCopyBatch = 8;           // loads in flight per thread in plain copies
constexpr uint32_t kStageBytes = 24576; // most input bytes one cone stages (prefetch registers: 96 B per thread)
constexpr uint32_t kStagePerThread = kStageBytes / kThreads;
constexpr uint32_t kRetrySlots = 64;    // failed attempts that run inside the tier launches

// 16 bytes as a native vector (stays in registers where a struct type may not)
typedef uint32_t vec16_t __attribute__((ext_vector_type(4)));

enum : uint32_t { kStOk = 0, kStRootFailed = 1, kStNoCleanSubtree = 2, kStBadFailureSet = 3 };

template <class T, int OP>
__device__ __forceinline__ T comb(T a, T b)
{
    if constexpr (OP == 0) return a + b; else return a | b;
}

// liveness of a LISTED process in a global round
__device__ __forceinline__ bool alive_at(uint32_t fail_round, uint32_t round)
{
    return fail_round != 0u && round < fail_round;
}

// The scenario's failure list, resolved for one attempt (root, first round).
struct FailTab {
    uint32_t n;            // slots
    uint32_t listed;       // slots in use
    uint32_t root_alive;   // the root is alive in the last round of the reduce
    uint32_t cnt_uc, cnt_tree;   // message counters of the workgroup
    uint32_t pad[3];
    uint32_t vr[16];       // virtual rank (kNoRank = unused slot)
    uint32_t fr[16];       // fail_round
    uint32_t row[16];      // row of the process (kNoRank: none)
    uint32_t idx[16];      // index inside its group
    uint32_t uc[16];       // up-correction rounds in which it still sends
    uint32_t tree[16];     // 1: it sends its tree message
};
static_assert(sizeof(FailTab) % 16 == 0, "FailTab must keep 16-byte alignment of what follows");

struct TierDesc {
    uint32_t dlo, dhi;          // depths of the rows this tier computes
    uint32_t child_in;          // 1: the tree messages of depth dhi+1 come from scratch
    uint32_t is_top;            // 1: dlo == 0, ends with the root's choice
    uint32_t in_off, in_meta_off;    // scratch offsets (bytes inside one scenario's scratch)
    uint32_t out_off, out_meta_off;
    uint32_t in_mask_off, out_mask_off;   // failure lists of the messages (16 bits per member), see process_lists
    uint32_t lds_rows;          // rows of LDS the tier stages
    uint32_t lds_bytes;         // dynamic LDS of the launch
    uint32_t kshift;            // a workgroup walks through 2^kshift consecutive cones
    uint32_t gshift;            // workgroups per scenario = 2^gshift = 2^(dlo - kshift)
    uint32_t threads;           // workgroup size of tier_kernel: 64, 128 or kThreads
};

struct RunArgs {
    Geom g;
    const unsigned char* payload;
    uint64_t scen_stride_bytes;
    const uint32_t* root;        // [S] or nullptr (reduce)
    const uint32_t* attempts;    // [S] or nullptr (allreduce: root = attempts - 1)
    const uint32_t* fail_rank;
    const uint32_t* fail_round;
    uint32_t* status;
    unsigned char* result;
    unsigned long long* msgs;
    uint32_t nmsg;               // counters per scenario: 2 (reduce) or 4 (allreduce)
    uint32_t S;
    unsigned char* ws;           // scratch
    uint64_t ws_stride;          // bytes per scenario (per workgroup in the retry kernel)
    uint32_t vroot_off;
    uint32_t vec16;              // 1: rows are 16-byte aligned in HBM: 16-byte staging
    uint32_t ntiers;
    uint32_t tier;               // tier run by this launch
    const uint32_t* retry_list;  // pairs (scenario, attempt) of attempts whose root had failed, or nullptr
    const uint32_t* retry_count; // entries in retry_list
    uint32_t retry_slots;        // entries run by the tier launches (the rest by the retry kernel)
    uint32_t lift;               // levels above the deepest tier that its kernel folds as well (eight lanes per subtree)
    uint32_t lift_off, lift_meta_off;   // where it leaves those rows' messages and words (inside a scenario's scratch)
    uint32_t pad0;
    unsigned char* retry_ws;     // scratch of the retry entries, ws_stride bytes each
    uint32_t* fix_list;          // four words per entry (scenario or S + retry entry, subtree, scenario, root):
    uint32_t* fix_count;         //   subtrees of the deepest tier that the general (LDS tile) kernel runs
    uint32_t* wfix_list;         // the same for the subtrees that the register kernel with failure handling runs:
    uint32_t* wfix_count;        //   [0] entries without rows on the deepest level, filled from the front of the
    uint32_t wfix_cap;           //   list, [1] entries with such rows, filled from its back (wfix_cap entries)
    uint32_t wave_general;       // 1: the listed subtrees go to wfix_list
    uint32_t info;               // 1: carry the lists of failed processes with the tree messages
    uint32_t* info_count;        // [S] or nullptr
    uint32_t* info_ids;          // [S][max(f,1)] or nullptr
    uint32_t* info_child;        // [S][W] or nullptr
    TierDesc tiers[kMaxTiers];
};

// One entry of the failure list, resolved by lane q < f of the first wavefront
// (the other lanes hold "unused"), plus the two facts about the whole list.
struct FailRegs {
    uint32_t vr, fr, row, idx, uc, tree;
    uint32_t listed, root_alive;
};

// Entry tid of the scenario's failure list as it stands in memory (unused for tid >= f).
struct FailRaw {
    uint32_t rank, round;
};

__device__ __forceinline__ FailRaw failtab_load(const Geom& g, const uint32_t* fail_rank, const uint32_t* fail_round,
                                                uint32_t s)
{
    const uint32_t F = g.f > 0 ? g.f : 1;
    FailRaw w;
    w.rank = kNoRank; w.round = 0;
    if (threadIdx.x < g.f) {
        w.rank = fail_rank[size_t(s) * F + threadIdx.x];
        w.round = fail_round[size_t(s) * F + threadIdx.x];
    }
    return w;
}

// called by the threads tid < 64 (one full wavefront, so that the ballots are defined)
__device__ __forceinline__ FailRegs failtab_compute(const Geom& g, const FailRaw& w, uint32_t root, uint32_t base)
{
    const uint32_t tid = threadIdx.x;
    FailRegs r;
    r.vr = kNoRank; r.fr = 0; r.row = kNoRank; r.idx = 0; r.uc = 0; r.tree = 0;
    if (tid < g.f) {
        uint32_t rank = w.rank;
        if (rank != kNoRank) {
            r.fr = w.round;
            r.vr = relabel(rank, root);
            uint32_t gs;
            if (r.vr == 0) {
                r.row = g.a > 1 ? g.M - 1 : kNoRank;
                r.idx = g.a - 1;
                gs = g.a;
            } else {
                uint32_t j = fdiv(r.vr - 1, g.divW);
                r.idx = r.vr - 1 - j * g.W;
                r.row = j;
                gs = group_size(g, j);
                r.tree = alive_at(r.fr, base + tree_send_round(g, r.idx, j)) ? 1u : 0u;
            }
            // the send of up-correction round t happens iff base + t < fr
            uint32_t done = r.fr > base + 1 ? r.fr - base - 1 : 0u;
            r.uc = done < gs - 1 ? done : gs - 1;
        }
    }
    unsigned long long m = __ballot(r.vr != kNoRank);
    unsigned long long rd = __ballot(r.vr == 0 && !alive_at(r.fr, base + g.Rred));
    r.listed = uint32_t(__popcll(m));
    r.root_alive = rd == 0ull ? 1u : 0u;
    return r;
}

// called by the same threads
__device__ __forceinline__ void failtab_store(FailTab& ft, const Geom& g, const FailRegs& r)
{
    const uint32_t tid = threadIdx.x;
    if (tid < 16) {
        ft.vr[tid] = r.vr; ft.fr[tid] = r.fr; ft.row[tid] = r.row; ft.idx[tid] = r.idx; ft.uc[tid] = r.uc;
        ft.tree[tid] = r.tree;
    }
    if (tid == 0) {
        ft.n = g.f;
        ft.cnt_uc = 0;
        ft.cnt_tree = 0;
        ft.listed = r.listed;
        ft.root_alive = r.root_alive;
    }
}

__device__ __forceinline__ void load_failtab(FailTab& ft, const Geom& g, const uint32_t* fail_rank,
                                             const uint32_t* fail_round, uint32_t s, uint32_t root,
                                             uint32_t base)
{
    if (threadIdx.x < 64) {
        const FailRaw w = failtab_load(g, fail_rank, fail_round, s);
        const FailRegs r = failtab_compute(g, w, root, base);
        failtab_store(ft, g, r);
    }
}

// One (row, value index) item: up-correction values of the W group members, tree
// messages of the row's members.  rows: LDS image of the cone, row stride W*E
// values; meta: per LDS row, bits 0..15 = member sent its tree message, bits
// 16..31 = failed bit of that message.
template <class T, int OP, int WP>
__device__ __forceinline__ void process_item(const Geom& g, const FailTab& ft, T* rows, uint32_t* meta,
                                             uint32_t li, uint32_t j, uint32_t e, bool kids_in_lds,
                                             bool check_fail, T* vroot_out, uint32_t& uc_cnt, uint32_t& tree_cnt)
{
    const uint32_t W = g.W, E = g.E, RE = W * E;
    const bool last = (j == g.M - 1);
    const uint32_t gs = (last && g.a > 1) ? g.a : W;      // group size, root included
    const uint32_t nk = last ? g.nlast : W;               // tree members of the row
    T* rp = rows + size_t(li) * RE + e;

    T x[WP];
#pragma unroll
    for (int w = 0; w < WP; ++w) x[w] = (uint32_t(w) < gs) ? rp[w * E] : T(0);

    // failures of this row: tl = packed 4-bit "rounds in which member w still sends"
    unsigned long long tl = 0x1111111111111111ull * (unsigned long long)(gs - 1);
    uint32_t sent = (1u << nk) - 1u;
    bool rowfail = false;
    if (check_fail) {
        for (uint32_t q = 0; q < ft.n; ++q) {
            if (ft.row[q] == j) {
                rowfail = true;
                uint32_t i4 = 4u * ft.idx[q];
                tl = (tl & ~(15ull << i4)) | ((unsigned long long)ft.uc[q] << i4);
                if (!ft.tree[q]) sent &= ~(1u << ft.idx[q]);
            }
        }
    }

    // up-correction: member i folds, in round order t = 1..gs-1, the input of
    // member (i - t) mod gs, if that member was alive in round t
    T v[WP];
    if (!rowfail) {
#pragma unroll
        for (int i = 0; i < WP; ++i) {
            T acc = x[i];
#pragma unroll
            for (int w = i - 1; w >= 0; --w) acc = comb<T, OP>(acc, x[w]);
#pragma unroll
            for (int w = WP - 1; w > i; --w)
                if (uint32_t(w) < gs) acc = comb<T, OP>(acc, x[w]);
            v[i] = acc;
        }
    } else {
#pragma unroll
        for (int i = 0; i < WP; ++i) {
            T acc = x[i];
#pragma unroll
            for (int w = i - 1; w >= 0; --w) {
                const uint32_t t = exchange_round(uint32_t(w), uint32_t(i), gs);
                if (t <= uint32_t((tl >> (4 * w)) & 15ull)) acc = comb<T, OP>(acc, x[w]);
            }
#pragma unroll
            for (int w = WP - 1; w > i; --w) {
                const uint32_t t = exchange_round(uint32_t(w), uint32_t(i), gs);
                if (uint32_t(w) < gs && t <= uint32_t((tl >> (4 * w)) & 15ull)) acc = comb<T, OP>(acc, x[w]);
            }
            v[i] = acc;
        }
    }

    if (last && g.a > 1 && vroot_out != nullptr) {
        // the root's value after its up-correction: member a-1 of the last group
        T vr = T(0);
#pragma unroll
        for (int k = 0; k < WP; ++k)
            if (uint32_t(k) == g.a - 1) vr = v[k];
        vroot_out[e] = vr;
    }

    // tree phase: add what the children sent (lower-numbered child first), set
    // the failed bit where a child's message is missing or carries the bit
    uint32_t flag = 0;
    if (kids_in_lds) {
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            uint32_t jc = 2u * j + 1u + uint32_t(c);
            if (jc < g.M) {
                uint32_t lc = 2u * li + 1u + uint32_t(c);
                uint32_t cm = meta[lc];
                uint32_t nkc = (jc == g.M - 1) ? g.nlast : W;
                uint32_t cmask = (1u << nkc) - 1u;
                const T* cp = rows + size_t(lc) * RE + e;
                if ((cm & cmask) == cmask) {
#pragma unroll
                    for (int k = 0; k < WP; ++k)
                        if (uint32_t(k) < nkc) v[k] = comb<T, OP>(v[k], cp[k * E]);
                } else {
#pragma unroll
                    for (int k = 0; k < WP; ++k)
                        if (uint32_t(k) < nkc && ((cm >> k) & 1u)) v[k] = comb<T, OP>(v[k], cp[k * E]);
                }
                flag |= ((cm >> 16) | ~cm) & cmask;
            }
        }
    }

#pragma unroll
    for (int k = 0; k < WP; ++k)
        if (uint32_t(k) < gs) rp[k * E] = v[k];

    if (e == 0) {
        meta[li] = (sent & 0xFFFFu) | (flag << 16);
        uint32_t c = 0;
        if (!rowfail) {
            c = gs * (gs - 1);
        } else {
#pragma unroll
            for (int w = 0; w < WP; ++w)
                if (uint32_t(w) < gs) c += uint32_t((tl >> (4 * w)) & 15ull);
        }
        uc_cnt += c;
        tree_cnt += uint32_t(__popc(sent));
    }
}

// The lists of failed processes the tree messages of one row carry (first scheme
// of section "Failure information"; the second scheme sends their length): lmask
// holds, per LDS row, W 16-bit words, a set of slots of the scenario's failure
// list (only listed processes ever fail to send).  A member adds the group mates
// whose up-correction message did not come, the children that sent nothing, and
// its children's lists.  Concatenated lists are disjoint, so the length is the
// number of bits.  Runs beside process_item on the same level: reads the children's
// meta words and lists, writes the row's lists.
__device__ __forceinline__ void process_lists(const Geom& g, const FailTab& ft, const uint32_t* meta, uint16_t* lmask,
                                              uint32_t li, uint32_t j, bool kids_in_lds, bool check_fail)
{
    const uint32_t W = g.W;
    const bool last = (j == g.M - 1);
    const uint32_t gs = (last && g.a > 1) ? g.a : W;      // group size, root included
    for (uint32_t i = 0; i < W; ++i) {
        uint32_t mk = 0;
        if (check_fail && i < gs) {
            // member i misses the message of listed member w, due in round t = (i - w) mod gs, iff w sends in
            // fewer rounds than t
            for (uint32_t q = 0; q < ft.n; ++q) {
                if (ft.row[q] != j || ft.idx[q] == i) continue;
                const uint32_t w = ft.idx[q];
                const uint32_t t = exchange_round(w, i, gs);
                if (t > ft.uc[q]) mk |= 1u << q;
            }
        }
        if (kids_in_lds) {
            for (uint32_t c = 0; c < 2; ++c) {
                const uint32_t jc = 2u * j + 1u + c;
                if (jc >= g.M) continue;
                const uint32_t lc = 2u * li + 1u + c;
                const uint32_t nkc = (jc == g.M - 1) ? g.nlast : W;
                if (i >= nkc) continue;
                if ((meta[lc] >> i) & 1u) {
                    mk |= lmask[size_t(lc) * W + i];               // the child's list
                } else {
                    for (uint32_t q = 0; q < ft.n; ++q)            // the child itself
                        if (ft.row[q] == jc && ft.idx[q] == i) mk |= 1u << q;
                }
            }
        }
        lmask[size_t(li) * W + i] = uint16_t(mk);
    }
}

// Workgroup barrier that orders LDS traffic only: prefetch loads of the next cone
// stay in flight across it (a full __syncthreads would wait for them).
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Copy `bytes` from src (HBM) to dst (LDS) in pieces of sizeof(V), kCopyBatch loads
// in flight per thread.
template <class V>
__device__ __forceinline__ void copy_to_lds(unsigned char* dst, const unsigned char* src, uint32_t bytes)
{
    const uint32_t n = bytes / uint32_t(sizeof(V));
    const uint32_t nthr = blockDim.x;
    for (uint32_t c0 = threadIdx.x; c0 < n; c0 += nthr * kCopyBatch) {
        V r[kCopyBatch];
#pragma unroll
        for (int u = 0; u < kCopyBatch; ++u) {
            uint32_t ci = c0 + uint32_t(u) * nthr;
            r[u] = reinterpret_cast<const V*>(src)[ci < n ? ci : 0u];    // always a valid address
        }
#pragma unroll
        for (int u = 0; u < kCopyBatch; ++u) {
            uint32_t ci = c0 + uint32_t(u) * nthr;
            if (ci < n) reinterpret_cast<V*>(dst)[ci] = r[u];
        }
    }
}

// Staging of a cone's inputs through registers, so that the loads of the next
// cone are in flight while the current one is reduced.
//
// The LDS image of a cone is contiguous: LDS row li at li * RB; LDS row li lies on
// level l = ilog2(li + 1) of the cone and is global row (r << l) + li, r = the
// cone's top row = 2^dlo - 1 + cone.  Global row jg starts at byte (1 + jg*W)*EB of
// the scenario's payload (virtual rank 1 + jg*W).  So the source offset of a chunk
// is  base + cone * step  with per-chunk constants base, step = RB << l.
// Rows >= M start at or beyond P*EB, so one clip against the payload size covers
// missing rows and the short last row.  Virtual rank `root` (when the root is not
// process 0) and the position virtual rank P would have (the root as member a-1 of
// the last group) are patched in afterwards.
template <class V>
struct Stage {
    static constexpr int NB = int(kStageBytes / (sizeof(V) * kThreads));
    V reg[NB];
    uint32_t base[NB];
    uint32_t step[NB];
    uint32_t okm_lo, okm_hi;      // chunk u was loaded

    __device__ __forceinline__ void init(const Geom& g, uint32_t dlo, uint32_t h)
    {
        const uint32_t CH = uint32_t(sizeof(V));
        const uint32_t n = (((2u << h) - 1u) * g.RB) / CH;
        const uint32_t top0 = (1u << dlo) - 1u;
#pragma unroll
        for (int u = 0; u < NB; ++u) {
            const uint32_t ci = threadIdx.x + uint32_t(u) * blockDim.x;
            uint32_t b = 0xFFFFFFFFu, st = 0u;         // never passes the clip
            if (ci < n) {
                const uint32_t off = ci * CH;
                const uint32_t li = fdiv(off, g.divRB);
                const uint32_t l = ilog2(li + 1u);
                b = (1u + ((top0 << l) + li) * g.W) * g.EB + (off - li * g.RB);
                st = g.RB << l;
            }
            base[u] = b;
            step[u] = st;
        }
        okm_lo = okm_hi = 0;
    }

    __device__ __forceinline__ void issue(const Geom& g, const unsigned char* pay, uint32_t cone, uint32_t root)
    {
        const uint32_t CH = uint32_t(sizeof(V));
        const uint32_t pay_bytes = g.P * g.EB;
        const uint32_t skip_lo = root != 0 ? root * g.EB : 0xFFFFFFFFu;
        unsigned long long okm = 0;
#pragma unroll
        for (int u = 0; u < NB; ++u) {
            const uint32_t sb = base[u] + cone * step[u];
            // base = 0xFFFFFFFF marks "no chunk"; real offsets stay below 2^32 - CH
            const bool ok = base[u] != 0xFFFFFFFFu && sb + CH <= pay_bytes && (sb - skip_lo >= g.EB);
            reg[u] = *reinterpret_cast<const V*>(pay + (ok ? sb : 0u));    // always a valid address
            okm |= (unsigned long long)(ok ? 1u : 0u) << u;
        }
        okm_lo = uint32_t(okm);
        okm_hi = uint32_t(okm >> 32);
    }

    __device__ __forceinline__ void commit(unsigned char* lrows) const
    {
        const uint32_t CH = uint32_t(sizeof(V));
        const unsigned long long okm = (unsigned long long)okm_lo | ((unsigned long long)okm_hi << 32);
#pragma unroll
        for (int u = 0; u < NB; ++u) {
            const uint32_t ci = threadIdx.x + uint32_t(u) * blockDim.x;
            if ((okm >> u) & 1ull) *reinterpret_cast<V*>(lrows + size_t(ci) * CH) = reg[u];
        }
    }
};

// LDS row of global row jr inside the cone with top row r and height h, or kNoRank
__device__ __forceinline__ uint32_t local_row(uint32_t jr, uint32_t r, uint32_t h)
{
    const uint32_t d = ilog2(jr + 1u), dr = ilog2(r + 1u);
    if (d < dr || d - dr > h || ((jr + 1u) >> (d - dr)) != r + 1u) return kNoRank;
    return jr - (r << (d - dr));
}

// Patches after commit(): disjoint LDS bytes, written by the first threads.
template <class V>
__device__ __forceinline__ void stage_patches(const Geom& g, unsigned char* lrows, const unsigned char* pay,
                                              uint32_t r, uint32_t h, uint32_t root)
{
    const uint32_t CH = uint32_t(sizeof(V));
    const uint32_t tid = threadIdx.x;
    if (root != 0) {          // virtual rank `root` is process 0
        const uint32_t jr = fdiv(root - 1u, g.divW);
        const uint32_t li = local_row(jr, r, h);
        if (li != kNoRank) {
            unsigned char* dst = lrows + size_t(li) * g.RB + (root - 1u - jr * g.W) * g.EB;
            for (uint32_t o = tid * CH; o < g.EB; o += blockDim.x * CH)
                *reinterpret_cast<V*>(dst + o) = *reinterpret_cast<const V*>(pay + o);
        }
    }
    if (g.a > 1) {            // the root as member a-1 of the last group
        const uint32_t li = local_row(g.M - 1u, r, h);
        if (li != kNoRank) {
            unsigned char* dst = lrows + size_t(li) * g.RB + (g.a - 1u) * g.EB;
            const unsigned char* src = pay + size_t(root) * g.EB;
            for (uint32_t o = tid * CH; o < g.EB; o += blockDim.x * CH)
                *reinterpret_cast<V*>(dst + o) = *reinterpret_cast<const V*>(src + o);
        }
    }
}

// The same two patches with the loads apart from the LDS stores (one chunk per
// thread: values of at most kThreads * sizeof(V) bytes).
template <class V>
struct PatchRegs {
    V a, b;
    uint32_t dst_a, dst_b;        // LDS byte offsets, kNoRank = none

    __device__ __forceinline__ void issue(const Geom& g, const unsigned char* pay, uint32_t r, uint32_t h, uint32_t root)
    {
        const uint32_t o = threadIdx.x * uint32_t(sizeof(V));
        dst_a = dst_b = kNoRank;
        if (root != 0) {
            const uint32_t jr = fdiv(root - 1u, g.divW);
            const uint32_t li = local_row(jr, r, h);
            if (li != kNoRank && o < g.EB) {
                dst_a = li * g.RB + (root - 1u - jr * g.W) * g.EB + o;
                a = *reinterpret_cast<const V*>(pay + o);
            }
        }
        if (g.a > 1) {
            const uint32_t li = local_row(g.M - 1u, r, h);
            if (li != kNoRank && o < g.EB) {
                dst_b = li * g.RB + (g.a - 1u) * g.EB + o;
                b = *reinterpret_cast<const V*>(pay + size_t(root) * g.EB + o);
            }
        }
    }
    __device__ __forceinline__ void commit(unsigned char* lrows) const
    {
        if (dst_a != kNoRank) *reinterpret_cast<V*>(lrows + dst_a) = a;
        if (dst_b != kNoRank) *reinterpret_cast<V*>(lrows + dst_b) = b;
    }
};

// does the cone (top row r, height h) hold a row with a listed process?
__device__ __forceinline__ bool cone_has_failure(const FailTab& ft, uint32_t r, uint32_t h)
{
    bool any = false;
    if (ft.listed != 0)
        for (uint32_t q = 0; q < ft.n; ++q)
            if (ft.row[q] != kNoRank && local_row(ft.row[q], r, h) != kNoRank) any = true;
    return any;
}

// The rounds of one staged cone, deepest level first, then the hand-over to the
// tier above or the root's choice.  LDS-only barriers; ends with one.
template <class T, int OP, int WP>
__device__ __forceinline__ void cone_rounds(const RunArgs& A, const TierDesc& td, const FailTab& ft, T* rows,
                                            uint32_t* lmeta, uint16_t* lmask, uint32_t s, uint32_t root, uint32_t cone,
                                            const unsigned char* pay, unsigned char* wsS, bool discard,
                                            uint32_t& uc_cnt, uint32_t& tree_cnt)
{
    const Geom& g = A.g;
    const uint32_t tid = threadIdx.x, nthr = blockDim.x;
    const uint32_t h = td.dhi - td.dlo;
    const uint32_t r = (1u << td.dlo) - 1u + cone;
    const bool check_fail = cone_has_failure(ft, r, h);
    T* vroot_out = reinterpret_cast<T*>(wsS + A.vroot_off);

    for (int l = int(h); l >= 0; --l) {
        const uint32_t lfirst = (1u << l) - 1u;
        const uint32_t gfirst = ((r + 1u) << l) - 1u;
        if (gfirst < g.M) {
            uint32_t cnt = g.M - gfirst;
            if (cnt > (1u << l)) cnt = 1u << l;
            const uint32_t nitems = cnt * g.E;
            const bool kids = (uint32_t(l) < h) || td.child_in;
            for (uint32_t it = tid; it < nitems; it += nthr) {
                const uint32_t lr = fdiv(it, g.divE);
                const uint32_t e = it - lr * g.E;
                process_item<T, OP, WP>(g, ft, rows, lmeta, lfirst + lr, gfirst + lr, e, kids, check_fail,
                                        vroot_out, uc_cnt, tree_cnt);
            }
            if (lmask != nullptr)
                for (uint32_t lr = tid; lr < cnt; lr += nthr)
                    process_lists(g, ft, lmeta, lmask, lfirst + lr, gfirst + lr, kids, check_fail);
        }
        lds_barrier();
    }

    if (!td.is_top) {
        unsigned char* dst = wsS + td.out_off + size_t(cone) * g.RB;
        if (A.vec16) {
            for (uint32_t o = tid * 16u; o < g.RB; o += nthr * 16u)
                *reinterpret_cast<vec16_t*>(dst + o) = *reinterpret_cast<const vec16_t*>(reinterpret_cast<unsigned char*>(rows) + o);
        } else {
            for (uint32_t o = tid; o < g.W * g.E; o += nthr) reinterpret_cast<T*>(dst)[o] = rows[o];
        }
        if (tid == 0) reinterpret_cast<uint32_t*>(wsS + td.out_meta_off)[cone] = lmeta[0];
        if (lmask != nullptr && tid < g.W)
            reinterpret_cast<uint16_t*>(wsS + td.out_mask_off)[size_t(cone) * g.W + tid] = lmask[tid];
    } else if (!discard) {
        // Algorithm "reduce at the root": lowest-numbered child whose message is
        // present and reports no failure; the root adds its own value iff that
        // subtree holds no member of the root's group (children a .. f+1).
        const uint32_t cm = lmeta[0];
        const uint32_t nk0 = row_members(g, 0);
        const uint32_t okm = cm & ~(cm >> 16) & ((1u << nk0) - 1u);
        uint32_t st = kStOk;
        if (!ft.root_alive) st = kStRootFailed;
        else if (okm == 0) st = kStNoCleanSubtree;
        T* res = reinterpret_cast<T*>(A.result) + size_t(s) * g.E;
        for (uint32_t e = tid; e < g.E; e += nthr) {
            T val = T(0);
            if (st == kStOk) {
                const uint32_t ks = uint32_t(__ffs(int(okm))) - 1u;
                val = rows[ks * g.E + e];
                if (ks + 1u >= g.a) {
                    T vr;
                    if (g.a == 1) vr = reinterpret_cast<const T*>(pay + size_t(root) * g.EB)[e];   // the root's input
                    else if (A.ntiers == 1) vr = rows[size_t(g.M - 1u) * g.W * g.E + (g.a - 1u) * g.E + e];
                    else vr = vroot_out[e];       // written by the deepest tier, an earlier launch
                    val = comb<T, OP>(vr, val);
                }
            }
            res[e] = val;
        }
        if (tid == 0) A.status[s] = st;
        if (A.info) {
            // what the root received from each child, and the list of the message it selected, as
            // slots of the failure list; the ranks themselves in slot order
            const uint32_t F = g.f > 0 ? g.f : 1;
            const uint32_t ks = st == kStOk ? uint32_t(__ffs(int(okm))) - 1u : 0u;
            const uint32_t sel = st == kStOk ? uint32_t(lmask[ks]) : 0u;
            if (A.info_child && tid < g.W) {
                uint32_t w = 0;
                if (st != kStRootFailed && tid < nk0) {
                    const uint32_t present = (cm >> tid) & 1u, fbit = (cm >> (16u + tid)) & 1u;
                    w = present ? ((fbit ? 2u : 1u) << 16) | uint32_t(lmask[tid]) : 0u;
                }
                A.info_child[size_t(s) * g.W + tid] = w;
            }
            if (A.info_count && tid == 0) A.info_count[s] = uint32_t(__popc(sel));
            if (A.info_ids && tid < F) {
                // the tid-th set bit of sel
                uint32_t rank = kNoRank, seen = 0;
                for (uint32_t q = 0; q < g.f; ++q)
                    if ((sel >> q) & 1u) {
                        if (seen == tid) rank = A.fail_rank[size_t(s) * F + q];
                        ++seen;
                    }
                A.info_ids[size_t(s) * F + tid] = rank;
            }
        }
    }
    lds_barrier();
}

// messages of the level below an upper tier's cone, from scratch into LDS
template <class T>
__device__ __forceinline__ void stage_children(const RunArgs& A, const TierDesc& td, unsigned char* lrows_b,
                                               uint32_t* lmeta, uint16_t* lmask, const unsigned char* wsS,
                                               uint32_t cone)
{
    const Geom& g = A.g;
    const uint32_t h = td.dhi - td.dlo;
    const uint32_t r = (1u << td.dlo) - 1u + cone;
    const uint32_t nx = (2u << h) - 1u;
    const uint32_t per = 2u << h;                       // rows of the level below, per cone
    const uint32_t first = ((r + 1u) << (h + 1)) - 1u;  // its first global row
    const uint32_t cc = first < g.M ? (g.M - first < per ? g.M - first : per) : 0u;
    const unsigned char* src = wsS + td.in_off + size_t(cone) * per * g.RB;
    if (A.vec16) copy_to_lds<vec16_t>(lrows_b + size_t(nx) * g.RB, src, cc * g.RB);
    else copy_to_lds<T>(lrows_b + size_t(nx) * g.RB, src, cc * g.RB);
    const uint32_t* msrc = reinterpret_cast<const uint32_t*>(wsS + td.in_meta_off) + size_t(cone) * per;
    for (uint32_t i = threadIdx.x; i < cc; i += blockDim.x) lmeta[nx + i] = msrc[i];
    if (lmask != nullptr) {
        const uint16_t* ksrc = reinterpret_cast<const uint16_t*>(wsS + td.in_mask_off) + size_t(cone) * per * g.W;
        for (uint32_t i = threadIdx.x; i < cc * g.W; i += blockDim.x) lmask[size_t(nx) * g.W + i] = ksrc[i];
    }
}

// A workgroup's walk through its cones of one tier of one (scenario, attempt).
template <class T, int OP, int WP, class V>
__device__ __forceinline__ void walk_cones(const RunArgs& A, const TierDesc& td, FailTab& ft, unsigned char* lrows,
                                           uint32_t* lmeta, uint32_t s, uint32_t root, uint32_t base,
                                           uint32_t c_lo, uint32_t c_hi, const unsigned char* pay,
                                           unsigned char* wsS, bool discard, uint32_t lds_rows_max)
{
    const Geom& g = A.g;
    const uint32_t h = td.dhi - td.dlo;
    // the lists of the staged rows sit behind the rows (16 bits per member)
    uint16_t* lmask = A.info ? reinterpret_cast<uint16_t*>(lrows + ((size_t(lds_rows_max) * g.RB + 15u) & ~size_t(15))) : nullptr;
    Stage<V> stg;
    stg.init(g, td.dlo, h);
    stg.issue(g, pay, c_lo, root);                 // in flight while the failure list is resolved
    load_failtab(ft, g, A.fail_rank, A.fail_round, s, root, base);
    uint32_t uc_cnt = 0, tree_cnt = 0;
    for (uint32_t cone = c_lo; cone < c_hi; ++cone) {
        const uint32_t r = (1u << td.dlo) - 1u + cone;
        stg.commit(lrows);
        stage_patches<V>(g, lrows, pay, r, h, root);
        if (td.child_in) stage_children<T>(A, td, lrows, lmeta, lmask, wsS, cone);
        __syncthreads();
        if (cone + 1 < c_hi) stg.issue(g, pay, cone + 1, root);    // prefetch
        cone_rounds<T, OP, WP>(A, td, ft, reinterpret_cast<T*>(lrows), lmeta, lmask, s, root, cone, pay, wsS, discard,
                               uc_cnt, tree_cnt);
    }
    if (A.msgs) {
        if (uc_cnt) atomicAdd(&ft.cnt_uc, uc_cnt);
        if (tree_cnt) atomicAdd(&ft.cnt_tree, tree_cnt);
        __syncthreads();
        if (threadIdx.x == 0) {
            if (ft.cnt_uc) atomicAdd(&A.msgs[size_t(s) * A.nmsg + 0], (unsigned long long)ft.cnt_uc);
            if (ft.cnt_tree) atomicAdd(&A.msgs[size_t(s) * A.nmsg + 1], (unsigned long long)ft.cnt_tree);
        }
    }
}

template <class T, int OP, int WP, bool VEC>
__global__ void __launch_bounds__(kThreads) tier_kernel(RunArgs A)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const TierDesc& td = A.tiers[A.tier];
    const uint32_t sv = blockIdx.x >> td.gshift;                      // scenario, or S + retry entry
    const uint32_t grp = blockIdx.x & ((1u << td.gshift) - 1u);
    uint32_t c_lo = grp << td.kshift;
    uint32_t c_hi = c_lo + (1u << td.kshift);
    const uint32_t top0 = (1u << td.dlo) - 1u;
    if (top0 + c_lo >= A.g.M) return;                                 // no such rows
    if (top0 + c_hi > A.g.M) c_hi = A.g.M - top0;

    uint32_t s = sv, root = 0, base = 0;
    bool discard = false;
    unsigned char* wsS;
    if (sv >= A.S) {
        // an attempt whose root had failed beforehand: messages are sent, nothing is delivered
        const uint32_t k = sv - A.S;
        uint32_t n = *A.retry_count;
        if (k >= n) return;
        s = A.retry_list[2u * k];
        root = A.retry_list[2u * k + 1u];
        base = root * A.g.Ratt;
        discard = true;
        wsS = A.retry_ws + size_t(k) * A.ws_stride;
    } else {
        if (A.status[s] == kStBadFailureSet) return;
        if (A.attempts) {
            root = A.attempts[s] - 1u;
            base = root * A.g.Ratt;
        } else if (A.root) {
            root = A.root[s];
        }
        wsS = A.ws + size_t(s) * A.ws_stride;
    }
    FailTab& ft = *reinterpret_cast<FailTab*>(smem);
    uint32_t* lmeta = reinterpret_cast<uint32_t*>(smem + sizeof(FailTab));
    unsigned char* lrows = smem + sizeof(FailTab) + ((size_t(td.lds_rows) * 4u + 15u) & ~size_t(15));
    const unsigned char* pay = A.payload + size_t(s) * A.scen_stride_bytes;
    if constexpr (VEC) walk_cones<T, OP, WP, vec16_t>(A, td, ft, lrows, lmeta, s, root, base, c_lo, c_hi, pay, wsS, discard, td.lds_rows);
    else walk_cones<T, OP, WP, T>(A, td, ft, lrows, lmeta, s, root, base, c_lo, c_hi, pay, wsS, discard, td.lds_rows);
}

// The deepest tier's subtrees that are not for the plain register kernel (failures,
// the short last group, ragged bottom level): workgroups stride over
// the list, one subtree at a time.  The entries are independent, so everything an
// entry needs from memory (its descriptor, the failure list, the rows, the two
// patched values) is requested while the entry before it is reduced out of LDS.
struct ListEntry {
    uint32_t sv, cone, s, root, base;
    bool valid, discard;
    unsigned char* wsS;
    const unsigned char* pay;
};

// entry i of the list: four words (scenario or S + retry entry, subtree, scenario, root), one load
__device__ __forceinline__ vec16_t list_load(const RunArgs& A, uint32_t i, uint32_t n)
{
    return reinterpret_cast<const vec16_t*>(A.fix_list)[i < n ? i : 0u];       // always a valid address
}

__device__ __forceinline__ ListEntry list_entry(const RunArgs& A, const vec16_t& w, bool valid)
{
    ListEntry en;
    en.valid = valid;
    en.sv = w.x; en.cone = w.y; en.s = w.z; en.root = w.w;
    en.discard = en.sv >= A.S;
    en.base = (en.discard || A.attempts) ? en.root * A.g.Ratt : 0u;
    en.wsS = en.discard ? A.retry_ws + size_t(en.sv - A.S) * A.ws_stride : A.ws + size_t(en.s) * A.ws_stride;
    en.pay = A.payload + size_t(en.s) * A.scen_stride_bytes;
    return en;
}

template <class T, int OP, int WP, bool VEC>
__global__ void __launch_bounds__(kThreads) tier_list_kernel(RunArgs A)
{
    using V = typename std::conditional<VEC, vec16_t, T>::type;
    extern __shared__ __align__(16) unsigned char smem[];
    const Geom& g = A.g;
    const TierDesc& td = A.tiers[0];
    FailTab& ft = *reinterpret_cast<FailTab*>(smem);
    uint32_t* lmeta = reinterpret_cast<uint32_t*>(smem + sizeof(FailTab));
    unsigned char* lrows = smem + sizeof(FailTab) + ((size_t(td.lds_rows) * 4u + 15u) & ~size_t(15));
    uint16_t* lmask = A.info ? reinterpret_cast<uint16_t*>(lrows + ((size_t(td.lds_rows) * g.RB + 15u) & ~size_t(15))) : nullptr;
    const uint32_t n = *A.fix_count;
    const uint32_t h = td.dhi - td.dlo;
    const uint32_t top0 = (1u << td.dlo) - 1u;
    const bool reg_patches = g.EB <= uint32_t(blockDim.x * sizeof(V));
    const uint32_t tid = threadIdx.x;
    const uint32_t stride = gridDim.x;
    if (blockIdx.x >= n) return;

    // Pipeline over the entries i, i + stride, ..: while entry i is reduced out of LDS, the rows, patches and
    // failure list of entry i + stride and the descriptor of entry i + 2 stride are on their way.
    Stage<V> stg;
    stg.init(g, td.dlo, h);
    PatchRegs<V> pr;
    pr.dst_a = pr.dst_b = kNoRank;
    ListEntry cur = list_entry(A, list_load(A, blockIdx.x, n), true);
    vec16_t nxt_w = list_load(A, blockIdx.x + stride, n);
    stg.issue(g, cur.pay, cur.cone, cur.root);
    if (reg_patches) pr.issue(g, cur.pay, top0 + cur.cone, h, cur.root);
    FailRaw raw = failtab_load(g, A.fail_rank, A.fail_round, cur.s);

    for (uint32_t i = blockIdx.x; i < n; i += stride) {
        __syncthreads();              // the previous entry is done with LDS
        if (tid < 64) failtab_store(ft, g, failtab_compute(g, raw, cur.root, cur.base));
        stg.commit(lrows);
        if (reg_patches) pr.commit(lrows);
        else stage_patches<V>(g, lrows, cur.pay, top0 + cur.cone, h, cur.root);
        __syncthreads();
        // Everything requested from here on is used after the rounds of this entry.  (Nothing is requested
        // before the waits above: they wait for all outstanding requests, loads and stores alike.)
        const vec16_t nxt2_w = list_load(A, i + 2u * stride, n);
        const ListEntry nxt = list_entry(A, nxt_w, i + stride < n);
        if (nxt.valid) {
            stg.issue(g, nxt.pay, nxt.cone, nxt.root);
            if (reg_patches) pr.issue(g, nxt.pay, top0 + nxt.cone, h, nxt.root);
            raw = failtab_load(g, A.fail_rank, A.fail_round, nxt.s);
        }
        uint32_t uc_cnt = 0, tree_cnt = 0;
        cone_rounds<T, OP, WP>(A, td, ft, reinterpret_cast<T*>(lrows), lmeta, lmask, cur.s, cur.root, cur.cone, cur.pay,
                               cur.wsS, cur.discard, uc_cnt, tree_cnt);
        if (A.msgs) {
            // per wavefront: sum over the lanes, one atomic each
#pragma unroll
            for (int d = 32; d >= 1; d >>= 1) {
                uc_cnt += __shfl_xor(uc_cnt, d);
                tree_cnt += __shfl_xor(tree_cnt, d);
            }
            if ((tid & 63u) == 0) {
                if (uc_cnt) atomicAdd(&A.msgs[size_t(cur.s) * A.nmsg + 0], (unsigned long long)uc_cnt);
                if (tree_cnt) atomicAdd(&A.msgs[size_t(cur.s) * A.nmsg + 1], (unsigned long long)tree_cnt);
            }
        }
        cur = nxt;
        nxt_w = nxt2_w;
    }
}

// launchers, one set per (value type, operator), defined in ftred_inst_*.hip
#define FTRED_DECLARE_LAUNCHERS(NAME)                                                         \
    hipError_t launch_tier_##NAME(const RunArgs& A, uint32_t grid, uint32_t lds, hipStream_t st); \
    hipError_t launch_list_##NAME(const RunArgs& A, uint32_t grid, uint32_t lds, hipStream_t st);

FTRED_DECLARE_LAUNCHERS(i64_sum)
FTRED_DECLARE_LAUNCHERS(i64_bor)
FTRED_DECLARE_LAUNCHERS(u32_sum)
FTRED_DECLARE_LAUNCHERS(u32_bor)
FTRED_DECLARE_LAUNCHERS(f64_sum)

#define FTRED_DEFINE_LAUNCHERS(NAME, T, OP)                                                        \
    template <int WP>                                                                              \
    static hipError_t tier_wp_##NAME(const RunArgs& A, uint32_t grid, uint32_t lds, hipStream_t st) \
    {                                                                                              \
        const uint32_t thr = A.tiers[A.tier].threads;                                              \
        if (A.vec16) hipLaunchKernelGGL((tier_kernel<T, OP, WP, true>), dim3(grid), dim3(thr), lds, st, A); \
        else hipLaunchKernelGGL((tier_kernel<T, OP, WP, false>), dim3(grid), dim3(thr), lds, st, A); \
        return hipGetLastError();                                                                  \
    }                                                                                              \
    template <int WP>                                                                              \
    static hipError_t list_wp_##NAME(const RunArgs& A, uint32_t grid, uint32_t lds, hipStream_t st) \
    {                                                                                              \
        const uint32_t thr = A.tiers[0].threads;                                                   \
        if (A.vec16) hipLaunchKernelGGL((tier_list_kernel<T, OP, WP, true>), dim3(grid), dim3(thr), lds, st, A); \
        else hipLaunchKernelGGL((tier_list_kernel<T, OP, WP, false>), dim3(grid), dim3(thr), lds, st, A);        \
        return hipGetLastError();                                                                  \
    }                                                                                              \
    hipError_t launch_list_##NAME(const RunArgs& A, uint32_t grid, uint32_t lds, hipStream_t st)    \
    {                                                                                              \
        switch (wp_bucket(A.g.W)) {                                                                \
            case 2: return list_wp_##NAME<2>(A, grid, lds, st);                                    \
            case 3: return list_wp_##NAME<3>(A, grid, lds, st);                                    \
            case 4: return list_wp_##NAME<4>(A, grid, lds, st);                                    \
            case 5: return list_wp_##NAME<5>(A, grid, lds, st);                                    \
            case 9: return list_wp_##NAME<9>(A, grid, lds, st);                                    \
            default: return list_wp_##NAME<16>(A, grid, lds, st);                                  \
        }                                                                                          \
    }                                                                                              \
    hipError_t launch_tier_##NAME(const RunArgs& A, uint32_t grid, uint32_t lds, hipStream_t st)    \
    {                                                                                              \
        switch (wp_bucket(A.g.W)) {                                                                \
            case 2: return tier_wp_##NAME<2>(A, grid, lds, st);                                    \
            case 3: return tier_wp_##NAME<3>(A, grid, lds, st);                                    \
            case 4: return tier_wp_##NAME<4>(A, grid, lds, st);                                    \
            case 5: return tier_wp_##NAME<5>(A, grid, lds, st);                                    \
            case 9: return tier_wp_##NAME<9>(A, grid, lds, st);                                    \
            default: return tier_wp_##NAME<16>(A, grid, lds, st);                                  \
        }                                                                                          \
    }

// compile-time group width the kernels are instantiated for: the smallest of
// {2,3,4,5,9,16} that holds W members
inline int wp_bucket(uint32_t W)
{
    if (W <= 2) return 2;
    if (W <= 3) return 3;
    if (W <= 4) return 4;
    if (W <= 5) return 5;
    if (W <= 9) return 9;
    return 16;
}

}  // namespace ftred

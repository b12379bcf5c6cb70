// Geometry of one plan and the rank -> partner index arithmetic, computed on the
// fly from the rank (no tables).  Used by the host (plan, ftred_partners) and by
// every kernel.
//
// Notation (paper: n processes, failure bound f):
//   P = n, W = f+1 (size of a full up-correction group = number of subtrees of
//   the root), E = values per process.
//   Virtual ranks: the root's number is swapped with 0 (section "Reduce").
//   A virtual rank v >= 1 is written v = 1 + j*W + i with
//     i = (v-1) mod W   subtree number k = i+1 (proof of the replication
//                       theorem: (a-1) mod (f+1) = k-1), and at the same time
//                       the index inside its up-correction group,
//     j = (v-1) div W   group number (section "Up-Correction") and at the same
//                       time the position inside subtree k.
//   "Row" j = the W consecutive ranks 1+j*W .. (j+1)*W = one up-correction
//   group = the j-th process of every subtree.  There are M = ceil((P-1)/W)
//   rows; the last one may be short, and then the root joins its group as the
//   member with index a-1, a = ((P-1) mod W) + 1: the position virtual rank P
//   would have.
//   Inside a subtree the processes form a binary heap on j (children of j are
//   2j+1 and 2j+2; process j = 0 is the child of the root).  A process sends its
//   tree message in round f + 1 + height.
//   The definition of the I(f)-tree leaves the shape inside a subtree free; a plan
//   can ask for another one (Geom::shape): k >= 3 children per process, filled
//   breadth-first (children of j are kj+1 .. kj+k), or the binomial tree built by
//   doubling (the parent of j >= 1 is j without its highest one bit; the children
//   of j are j + 2^b for every b above j's highest one bit).  The sh_* functions
//   below work for every shape; the kernels of the default shape use the faster
//   binary-heap forms.
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#define FT_HD __host__ __device__ __forceinline__
#else
#define FT_HD inline
#endif

namespace ftred {

constexpr uint32_t kNoRank = 0xFFFFFFFFu;
constexpr uint32_t kMaxF = 15;          // W <= 16: per-row member masks fit 16 bits

// floor(n / d) for any uint32 n, d >= 1, by multiply-high (Granlund & Montgomery)
struct FastDiv {
    uint32_t d, m, s1, s2;
};

inline FastDiv make_fastdiv(uint32_t d)
{
    FastDiv r;
    uint32_t l = 0;
    while ((uint64_t(1) << l) < d) ++l;          // ceil(log2 d)
    r.d = d;
    r.m = uint32_t((((uint64_t(1) << l) - d) << 32) / d + 1);
    r.s1 = l < 1 ? l : 1;
    r.s2 = l - r.s1;
    return r;
}

FT_HD uint32_t ft_mulhi(uint32_t a, uint32_t b)
{
#if defined(__HIP_DEVICE_COMPILE__)
    return __umulhi(a, b);
#else
    return uint32_t((uint64_t(a) * uint64_t(b)) >> 32);
#endif
}

FT_HD uint32_t fdiv(uint32_t n, const FastDiv& f)
{
    uint32_t q = ft_mulhi(f.m, n);
    return (((n - q) >> f.s1) + q) >> f.s2;
}

FT_HD uint32_t ilog2(uint32_t x)          // floor(log2 x), x >= 1
{
#if defined(__HIP_DEVICE_COMPILE__)
    return 31u - uint32_t(__clz(int(x)));
#else
    return 31u - uint32_t(__builtin_clz(x));
#endif
}

constexpr uint32_t kShapeBinomial = 1, kShapeBinary = 2, kShapeMaxArity = 64;

struct Geom {
    uint32_t P, f, W, E;
    uint32_t shape;      // tree inside a subtree: 2 = binary heap (default), k >= 3 = k-ary heap, 1 = binomial
    uint32_t esz;        // bytes of one value
    uint32_t EB;         // bytes of one process's payload = E * esz
    uint32_t RB;         // bytes of one row = W * EB
    uint32_t M;          // rows
    uint32_t a;          // ((P-1) mod W) + 1; the root is in a group iff a > 1
    uint32_t nlast;      // tree members of the last row (W if it is full)
    uint32_t L;          // floor(log2 M): depth of the deepest row (row 0 has depth 0)
    uint32_t D;          // height of the root = L + 1
    uint32_t Rred;       // rounds of one reduce = f + D
    uint32_t Ratt;       // rounds of one allreduce attempt = 2 (f + D)
    FastDiv divW, divE, divRB, divEB;
};

FT_HD uint32_t sh_height_m(uint32_t shape, uint32_t m, uint32_t j);

inline Geom make_geom(uint32_t P, uint32_t f, uint32_t E, uint32_t esz, uint32_t shape = kShapeBinary)
{
    Geom g;
    g.P = P; g.f = f; g.W = f + 1; g.E = E; g.esz = esz;
    g.shape = shape;
    g.EB = E * esz;
    g.RB = g.W * g.EB;
    g.M = (P - 1 + g.W - 1) / g.W;
    g.a = (P - 1) % g.W + 1;
    g.nlast = g.a == 1 ? g.W : g.a - 1;
    g.L = ilog2(g.M);
    g.D = g.L + 1;
    if (shape != kShapeBinary) g.D = 1 + sh_height_m(shape, g.M, 0);     // the largest subtree has M processes
    g.Rred = f + g.D;
    g.Ratt = 2 * g.Rred;
    g.divW = make_fastdiv(g.W);
    g.divE = make_fastdiv(E);
    g.divRB = make_fastdiv(g.RB);
    g.divEB = make_fastdiv(g.EB);
    return g;
}

// swap of the root's number with 0; the map is its own inverse
FT_HD uint32_t relabel(uint32_t rank, uint32_t root)
{
    return rank == root ? 0u : (rank == 0u ? root : rank);
}

// number of processes of the subtree with 0-based number i
FT_HD uint32_t subtree_size(const Geom& g, uint32_t i)
{
    return g.M - (i >= g.nlast ? 1u : 0u);
}

// tree members of row j (the last row may be short)
FT_HD uint32_t row_members(const Geom& g, uint32_t j)
{
    return j == g.M - 1 ? g.nlast : g.W;
}

// size of the up-correction group of row j, the root counted if it is a member
FT_HD uint32_t group_size(const Geom& g, uint32_t j)
{
    return (j == g.M - 1 && g.a > 1) ? g.a : g.W;
}

// Who exchanges with whom inside a group of gs members (up-correction of the reduce, correction rounds of the
// broadcast; sections "Reduce / Algorithm" and "Allreduce"): in round t = 1 .. gs - 1 member i sends to member
// exchange_target and hears from member exchange_source; the message of member w is due at member i in round
// exchange_round.  Every kernel takes the pairing from here, so another correction scheme replaces these four.
FT_HD constexpr uint32_t exchange_target(uint32_t i, uint32_t t, uint32_t gs) { return (i + t) % gs; }
FT_HD constexpr uint32_t exchange_source(uint32_t i, uint32_t t, uint32_t gs) { return (i + gs - t) % gs; }
FT_HD constexpr uint32_t exchange_round(uint32_t w, uint32_t i, uint32_t gs) { return w < i ? i - w : i + gs - w; }
// the same for a whole group: bit i of the result is set iff the member that sends to i in round t is in `senders`
FT_HD constexpr uint32_t exchange_targets(uint32_t senders, uint32_t t, uint32_t gs, uint32_t full)
{
    return ((senders << t) | (senders >> (gs - t))) & full;
}

// height of process (subtree i, position j) above the leaves of its subtree:
// the largest h with (j+1) * 2^h <= size of the subtree
FT_HD uint32_t height_of(const Geom& g, uint32_t i, uint32_t j)
{
    uint32_t m = subtree_size(g, i);
    uint32_t h = ilog2(m) - ilog2(j + 1);
    if (((j + 1) << h) > m) --h;
    return h;
}

FT_HD uint32_t sh_height(const Geom& g, uint32_t i, uint32_t j);

// round (1-based, inside one reduce) in which the process sends to its parent
FT_HD uint32_t tree_send_round(const Geom& g, uint32_t i, uint32_t j)
{
    return g.f + 1 + sh_height(g, i, j);
}

// depth below the root (children of the root have depth 1)
FT_HD uint32_t depth_of(uint32_t j)
{
    return 1 + ilog2(j + 1);
}

// is position jq a proper ancestor of position j (same subtree)?
FT_HD bool is_proper_ancestor(uint32_t jq, uint32_t j)
{
    uint32_t dq = ilog2(jq + 1), d = ilog2(j + 1);
    return d > dq && ((j + 1) >> (d - dq)) == jq + 1;
}

// ---------------------------------------------------------------------------
// the same questions for any shape of the tree inside a subtree (positions j of a subtree of m processes)

// height of position j: the longest chain of children below it
FT_HD uint32_t sh_height_m(uint32_t shape, uint32_t m, uint32_t j)
{
    uint32_t h = 0;
    if (shape == kShapeBinomial) {
        // children add one bits above j's highest one: the longest chain adds the lowest of them one by one,
        // j + (2^t - 1) 2^b0 must stay below m
        const uint32_t b0 = j == 0 ? 0u : ilog2(j) + 1u;
        while (b0 + h < 32u && uint64_t(j) + (((uint64_t(2) << h) - 1u) << b0) <= uint64_t(m) - 1u) ++h;
        return h;
    }
    uint64_t c = j;                          // the first child, the first child of that, ..
    while (c * shape + 1u < m) { c = c * shape + 1u; ++h; }
    return h;
}

FT_HD uint32_t sh_height(const Geom& g, uint32_t i, uint32_t j)
{
    return g.shape == kShapeBinary ? height_of(g, i, j) : sh_height_m(g.shape, subtree_size(g, i), j);
}

// depth below the root (the first process of a subtree has depth 1)
FT_HD uint32_t sh_depth(const Geom& g, uint32_t j)
{
    if (g.shape == kShapeBinary) return depth_of(j);
    if (g.shape == kShapeBinomial) {
#if defined(__HIP_DEVICE_COMPILE__)
        return 1u + uint32_t(__popc(j));
#else
        return 1u + uint32_t(__builtin_popcount(j));
#endif
    }
    uint32_t d = 1;
    uint64_t first = 0, count = 1;           // positions of the current level
    while (j >= first + count) { first += count; count *= g.shape; ++d; }
    return d;
}

// position of the parent of position j >= 1
FT_HD uint32_t sh_parent(const Geom& g, uint32_t j)
{
    if (g.shape == kShapeBinomial) return j - (1u << ilog2(j));
    return (j - 1u) / g.shape;
}

// fn(position) for every child of position j in a subtree of m processes, in ascending order
template <class Fn>
FT_HD void sh_for_children(const Geom& g, uint32_t m, uint32_t j, Fn fn)
{
    if (g.shape == kShapeBinomial) {
        for (uint32_t b = j == 0 ? 0u : ilog2(j) + 1u; b < 32u; ++b) {
            const uint64_t c = uint64_t(j) + (uint64_t(1) << b);
            if (c >= m) break;
            fn(uint32_t(c));
        }
    } else {
        for (uint32_t k = 1; k <= g.shape; ++k) {
            const uint64_t c = uint64_t(j) * g.shape + k;
            if (c >= m) break;
            fn(uint32_t(c));
        }
    }
}

// is position jq a proper ancestor of position j (same subtree)?  Parents have smaller positions.
FT_HD bool sh_is_proper_ancestor(const Geom& g, uint32_t jq, uint32_t j)
{
    if (g.shape == kShapeBinary) return is_proper_ancestor(jq, j);
    if (j <= jq) return false;
    while (j > jq) j = sh_parent(g, j);
    return j == jq;
}

// failure-free message counts (theorem on the number of messages)
inline uint64_t msgs_uc_ff(const Geom& g)
{
    return uint64_t(g.f) * g.W * ((g.P - 1) / g.W) + uint64_t(g.a) * (g.a - 1);
}

}  // namespace ftred

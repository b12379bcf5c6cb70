// Up-correction phase, tree phase and the root's choice for the other shapes of
// the tree inside a subtree of the root (k children per process, binomial): the
// definition of the I(f)-tree leaves that shape free, and the shape decides the
// number of rounds, which is what the latency question is about.
//
// The kernels of the default shape are built around the binary heap (cones of
// rows in LDS, post-order walks in registers).  These are plain instead: one
// launch per depth of the tree, deepest first; one thread per (row, value index)
// reads the W inputs of its row from HBM, forms the up-correction values in round
// order (Algorithm "Up-correction"), adds the tree messages of its children rows
// (Algorithm "reduce at non-roots"), which an earlier launch left in a scratch
// area in HBM, [row][member][value index] with one word of sent / failed bits per
// row (section "Failure information", third scheme), and leaves its own there.
// A last small launch is the root's choice (Algorithm "reduce at the root").  The
// scratch area is as large as the payload: this path is for comparing shapes, not
// for the benchmark.  Attempts of an allreduce whose root had failed deliver
// nothing; only their messages count, and those follow from the failure list
// alone (retry_counts_kernel).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ftred_geom.h"
#include "ftred_kernels.h"

namespace ftred {

struct ShapeLevel {
    uint32_t depth;            // depth of the rows of this launch (the first row of a subtree has depth 1)
    uint32_t j_lo, j_hi;       // candidate rows
    uint32_t filter;           // 1: only the rows of that depth among them (binomial: they do not form a range)
    uint32_t blocks_per_scen;
    FastDiv div_bps;
    uint32_t msg_off, meta_off;   // inside one scenario's scratch
};

template <class T, int OP, int WP>
__global__ void __launch_bounds__(256) shape_level_kernel(RunArgs A, ShapeLevel lv)
{
    __shared__ FailTab ft;
    __shared__ uint32_t cnt[2];
    const Geom& g = A.g;
    const uint32_t tid = threadIdx.x;
    const uint32_t s = fdiv(blockIdx.x, lv.div_bps);
    const uint32_t b = blockIdx.x - s * lv.blocks_per_scen;
    if (A.status[s] == kStBadFailureSet) return;
    uint32_t root = 0, base = 0;
    if (A.attempts) {
        root = A.attempts[s] - 1u;               // roots tried; the last one is alive
        base = root * g.Ratt;
    } else if (A.root) {
        root = A.root[s];
    }
    if (tid < 2) cnt[tid] = 0;
    load_failtab(ft, g, A.fail_rank, A.fail_round, s, root, base);
    __syncthreads();

    const uint32_t W = g.W, E = g.E, RE = W * E;
    const uint32_t it = b * 256u + tid;
    const uint32_t r = fdiv(it, g.divE);
    const uint32_t e = it - r * E;
    const uint32_t j = lv.j_lo + r;
    const bool valid = j < lv.j_hi && (!lv.filter || sh_depth(g, j) == lv.depth);
    uint32_t uc_cnt = 0, tree_cnt = 0;
    if (valid) {
        const T* pay = reinterpret_cast<const T*>(A.payload + size_t(s) * A.scen_stride_bytes);
        unsigned char* wsS = A.ws + size_t(s) * A.ws_stride;
        T* msg = reinterpret_cast<T*>(wsS + lv.msg_off);
        uint32_t* meta = reinterpret_cast<uint32_t*>(wsS + lv.meta_off);
        const bool last = j == g.M - 1u;
        const uint32_t gs = (last && g.a > 1) ? g.a : W;      // group size, the root included if it is a member
        const uint32_t nk = last ? g.nlast : W;               // tree members of the row

        // the inputs of the group: the row's members; the root as member a-1 of a short last group; the process
        // that carries the root's number is process 0 (the root swaps numbers with it)
        T x[WP];
#pragma unroll
        for (int w = 0; w < WP; ++w) {
            x[w] = T(0);
            if (uint32_t(w) < nk) x[w] = pay[(size_t(1u + j * W) + uint32_t(w)) * E + e];
            else if (uint32_t(w) < gs) x[w] = pay[size_t(root) * E + e];
        }
        if (root != 0) {
            const uint32_t jx = fdiv(root - 1u, g.divW), kx = root - 1u - jx * W;
            if (j == jx) {
                const T x0 = pay[e];
#pragma unroll
                for (int w = 0; w < WP; ++w) x[w] = uint32_t(w) == kx ? x0 : x[w];
            }
        }
        // failures of this row: tl = packed 4-bit "rounds in which member w still sends"
        unsigned long long tl = 0x1111111111111111ull * (unsigned long long)(gs - 1u);
        uint32_t sent = (1u << nk) - 1u;
        if (ft.listed != 0)
            for (uint32_t q = 0; q < ft.n; ++q)
                if (ft.row[q] == j) {
                    const uint32_t i4 = 4u * ft.idx[q];
                    tl = (tl & ~(15ull << i4)) | ((unsigned long long)ft.uc[q] << i4);
                    if (!ft.tree[q]) sent &= ~(1u << ft.idx[q]);
                }
        // up-correction: member i folds, in round order t = 1..gs-1, the input of member (i - t) mod gs, if that
        // member still sends in round t
        T v[WP];
#pragma unroll
        for (int i = 0; i < WP; ++i) {
            T acc = x[i];
#pragma unroll
            for (int w = i - 1; w >= 0; --w)
                if (exchange_round(uint32_t(w), uint32_t(i), gs) <= uint32_t((tl >> (4 * w)) & 15ull))
                    acc = comb<T, OP>(acc, x[w]);
#pragma unroll
            for (int w = WP - 1; w > i; --w)
                if (uint32_t(w) < gs &&
                    exchange_round(uint32_t(w), uint32_t(i), gs) <= uint32_t((tl >> (4 * w)) & 15ull))
                    acc = comb<T, OP>(acc, x[w]);
            v[i] = acc;
        }
        if (last && g.a > 1) {          // the root's value after its up-correction
            T vr = T(0);
#pragma unroll
            for (int k = 0; k < WP; ++k) vr = uint32_t(k) == g.a - 1u ? v[k] : vr;
            reinterpret_cast<T*>(wsS + A.vroot_off)[e] = vr;
        }
        // tree phase: the children's messages, lower-numbered child first; a missing message or one with the
        // failed bit sets the failed bit
        uint32_t flag = 0;
        sh_for_children(g, g.M, j, [&](uint32_t jc) {
            const uint32_t cm = meta[jc];
            const uint32_t nkc = jc == g.M - 1u ? g.nlast : W;
            const uint32_t cmask = (1u << nkc) - 1u;
            const T* cp = msg + size_t(jc) * RE + e;
#pragma unroll
            for (int k = 0; k < WP; ++k)
                if (uint32_t(k) < nkc && ((cm >> k) & 1u)) v[k] = comb<T, OP>(v[k], cp[size_t(k) * E]);
            flag |= ((cm >> 16) | ~cm) & cmask;
        });
        T* mp = msg + size_t(j) * RE + e;
#pragma unroll
        for (int k = 0; k < WP; ++k)
            if (uint32_t(k) < nk) mp[size_t(k) * E] = v[k];
        if (e == 0) {
            meta[j] = (sent & 0xFFFFu) | (flag << 16);
#pragma unroll
            for (int w = 0; w < WP; ++w)
                if (uint32_t(w) < gs) uc_cnt += uint32_t((tl >> (4 * w)) & 15ull);
            tree_cnt = uint32_t(__popc(sent));
        }
    }
    if (A.msgs) {
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) {
            uc_cnt += __shfl_xor(uc_cnt, d);
            tree_cnt += __shfl_xor(tree_cnt, d);
        }
        if ((tid & 63u) == 0) {
            if (uc_cnt) atomicAdd(&cnt[0], uc_cnt);
            if (tree_cnt) atomicAdd(&cnt[1], tree_cnt);
        }
        __syncthreads();
        if (tid == 0) {
            if (cnt[0]) atomicAdd(&A.msgs[size_t(s) * A.nmsg + 0], (unsigned long long)cnt[0]);
            if (cnt[1]) atomicAdd(&A.msgs[size_t(s) * A.nmsg + 1], (unsigned long long)cnt[1]);
        }
    }
}

// Algorithm "reduce at the root": lowest-numbered child whose message is present and reports no failure; the
// root adds its own value iff that subtree holds no member of the root's group (children a .. f+1).
template <class T, int OP>
__global__ void __launch_bounds__(64) shape_root_kernel(RunArgs A, uint32_t msg_off, uint32_t meta_off)
{
    const Geom& g = A.g;
    const uint32_t s = blockIdx.x, tid = threadIdx.x;
    if (A.status[s] == kStBadFailureSet) return;
    uint32_t root = 0, base = 0;
    if (A.attempts) {
        root = A.attempts[s] - 1u;
        base = root * g.Ratt;
    } else if (A.root) {
        root = A.root[s];
    }
    const uint32_t F = g.f > 0 ? g.f : 1;
    bool root_alive = true;
    for (uint32_t q = 0; q < g.f; ++q)
        if (A.fail_rank[size_t(s) * F + q] == root) root_alive = alive_at(A.fail_round[size_t(s) * F + q], base + g.Rred);
    const unsigned char* wsS = A.ws + size_t(s) * A.ws_stride;
    const T* row0 = reinterpret_cast<const T*>(wsS + msg_off);
    const uint32_t cm = reinterpret_cast<const uint32_t*>(wsS + meta_off)[0];
    const uint32_t okm = cm & ~(cm >> 16) & ((1u << row_members(g, 0)) - 1u);
    uint32_t st = kStOk;
    if (!root_alive) st = kStRootFailed;
    else if (okm == 0) st = kStNoCleanSubtree;
    const T* pay = reinterpret_cast<const T*>(A.payload + size_t(s) * A.scen_stride_bytes);
    const T* vroot = reinterpret_cast<const T*>(wsS + A.vroot_off);
    T* res = reinterpret_cast<T*>(A.result) + size_t(s) * g.E;
    for (uint32_t e = tid; e < g.E; e += 64u) {
        T val = T(0);
        if (st == kStOk) {
            const uint32_t ks = uint32_t(__ffs(int(okm))) - 1u;
            val = row0[size_t(ks) * g.E + e];
            if (ks + 1u >= g.a) val = comb<T, OP>(g.a == 1 ? pay[size_t(root) * g.E + e] : vroot[e], val);
        }
        res[e] = val;
    }
    if (tid == 0) A.status[s] = st;
}

// Messages of attempts whose root had failed beforehand (entries `first`, first + 1, .. of the retry list): such an
// attempt delivers nothing, and every process that is alive sends what it would send anyway (a reduce does not
// wait for what it receives), so the counts follow from the failure list: the failure-free counts (message-count
// theorem) less what each listed process no longer sends.
static __global__ void __launch_bounds__(256) retry_counts_kernel(RunArgs A, unsigned long long uc_ff, uint32_t first)
{
    const Geom& g = A.g;
    const uint32_t k = first + blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= *A.retry_count || !A.msgs) return;
    const uint32_t s = A.retry_list[2u * k], root = A.retry_list[2u * k + 1u];
    const uint32_t base = root * g.Ratt;
    const uint32_t F = g.f > 0 ? g.f : 1;
    unsigned long long uc = uc_ff, tree = g.P - 1u;
    for (uint32_t q = 0; q < g.f; ++q) {
        const uint32_t rank = A.fail_rank[size_t(s) * F + q];
        if (rank == kNoRank) continue;
        const uint32_t fr = A.fail_round[size_t(s) * F + q];
        const uint32_t vr = relabel(rank, root);
        uint32_t gs;
        if (vr == 0) {
            gs = g.a > 1 ? g.a : 1u;
        } else {
            const uint32_t j = fdiv(vr - 1u, g.divW);
            gs = group_size(g, j);
            if (!alive_at(fr, base + tree_send_round(g, vr - 1u - j * g.W, j))) tree -= 1u;
        }
        const uint32_t done = fr > base + 1u ? fr - base - 1u : 0u;      // up-correction rounds in which it still sends
        uc -= (gs - 1u) - (done < gs - 1u ? done : gs - 1u);
    }
    atomicAdd(&A.msgs[size_t(s) * A.nmsg + 0], uc);
    atomicAdd(&A.msgs[size_t(s) * A.nmsg + 1], tree);
}

#define FTRED_DECLARE_SHAPE_LAUNCHER(NAME) \
    hipError_t launch_shape_level_##NAME(const RunArgs& A, const ShapeLevel& lv, uint32_t grid, hipStream_t st); \
    hipError_t launch_shape_root_##NAME(const RunArgs& A, uint32_t msg_off, uint32_t meta_off, uint32_t grid, hipStream_t st);

FTRED_DECLARE_SHAPE_LAUNCHER(i64_sum)
FTRED_DECLARE_SHAPE_LAUNCHER(i64_bor)
FTRED_DECLARE_SHAPE_LAUNCHER(u32_sum)
FTRED_DECLARE_SHAPE_LAUNCHER(u32_bor)
FTRED_DECLARE_SHAPE_LAUNCHER(f64_sum)

#define FTRED_DEFINE_SHAPE_LAUNCHER(NAME, T, OP)                                                       \
    template <int WP>                                                                                  \
    static hipError_t shape_wp_##NAME(const RunArgs& A, const ShapeLevel& lv, uint32_t grid, hipStream_t st) \
    {                                                                                                  \
        hipLaunchKernelGGL((shape_level_kernel<T, OP, WP>), dim3(grid), dim3(256), 0, st, A, lv);       \
        return hipGetLastError();                                                                      \
    }                                                                                                  \
    hipError_t launch_shape_level_##NAME(const RunArgs& A, const ShapeLevel& lv, uint32_t grid, hipStream_t st) \
    {                                                                                                  \
        switch (wp_bucket(A.g.W)) {                                                                    \
            case 2: return shape_wp_##NAME<2>(A, lv, grid, st);                                        \
            case 3: return shape_wp_##NAME<3>(A, lv, grid, st);                                        \
            case 4: return shape_wp_##NAME<4>(A, lv, grid, st);                                        \
            case 5: return shape_wp_##NAME<5>(A, lv, grid, st);                                        \
            case 9: return shape_wp_##NAME<9>(A, lv, grid, st);                                        \
            default: return shape_wp_##NAME<16>(A, lv, grid, st);                                      \
        }                                                                                              \
    }                                                                                                  \
    hipError_t launch_shape_root_##NAME(const RunArgs& A, uint32_t msg_off, uint32_t meta_off, uint32_t grid, hipStream_t st) \
    {                                                                                                  \
        hipLaunchKernelGGL((shape_root_kernel<T, OP>), dim3(grid), dim3(64), 0, st, A, msg_off, meta_off); \
        return hipGetLastError();                                                                      \
    }

}  // namespace ftred

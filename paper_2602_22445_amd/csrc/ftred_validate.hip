// ftred_validate: checks results against the semantics, independently of the
// protocol kernels.  Sections "Reduce / Semantics" (items 3 and 4) and
// "Allreduce / Semantics" (items 4 and 5): the result must be the reduction over
// the never-failed processes combined with ONE subset of the processes that
// failed during the operation; every never-failed process of an allreduce holds
// it.  The message counters must lie in the range the message-count theorems
// allow (failed processes send fewer messages, nobody sends more).
//
// Pass 1 (one workgroup per chunk of ranks): partial reduction of the
// never-failed inputs, partial sums of |x| (tolerance scale for FTRED_F64), and
// the holder check of the chunk.  Pass 2 (one workgroup per scenario): partials
// folded in chunk order, subsets enumerated, status and counters checked.
#include <hip/hip_runtime.h>

#include <string.h>

#include <type_traits>

#include "../../include/ftred.h"
#include "ftred_plan.h"

using namespace ftred;

namespace {

struct ValArgs {
    Geom g;
    int kind;                       // 0 reduce, 1 allreduce
    uint32_t S;
    const uint32_t* root;           // reduce: [S] or nullptr
    const unsigned char* payload;
    uint64_t scen_stride_bytes;
    const uint32_t* fail_rank;
    const uint32_t* fail_round;
    const unsigned char* result;
    const uint32_t* has_bitmap;     // or nullptr
    const unsigned char* out;       // or nullptr
    const uint32_t* status;
    const uint32_t* attempts;       // or nullptr
    const unsigned long long* msgs; // or nullptr
    uint32_t* verdict;
    unsigned char* partial;         // [S][nchunks][E] values (8 bytes each)
    double* scale;                  // [S][nchunks][E]
    unsigned long long* n_invalid;  // device counter
    uint32_t chunk, nchunks;
    FastDiv div_nchunks;
    uint64_t uc_ff;                 // failure-free up-correction messages
};

template <class T, int OP>
__device__ __forceinline__ T vcomb(T a, T b)
{
    if constexpr (OP == 0) return a + b; else return a | b;
}

template <class T>
__device__ __forceinline__ bool same_bits(T a, T b)
{
    if constexpr (sizeof(T) == 8) return __builtin_bit_cast(unsigned long long, a) == __builtin_bit_cast(unsigned long long, b);
    else return __builtin_bit_cast(uint32_t, a) == __builtin_bit_cast(uint32_t, b);
}

__global__ void val_init_kernel(uint32_t S, uint32_t* verdict, unsigned long long* n_invalid)
{
    const uint32_t s = blockIdx.x * blockDim.x + threadIdx.x;
    if (s < S) verdict[s] = 0u;
    if (s == 0) *n_invalid = 0ull;
}

// failure list of the scenario in LDS: physical ranks
struct ValFail {
    uint32_t listed;
    uint32_t pad[3];
    uint32_t rank[16], round[16];
};

// V values per load (V * sizeof(T) = 16 bytes, or V = 1): streaming loads that
// bypass nothing but are marked non-temporal, the data is read once
template <class T, int V>
__device__ __forceinline__ void load_values(const T* p, T (&v)[V])
{
    if constexpr (V == 1) {
        v[0] = __builtin_nontemporal_load(p);
    } else {
        static_assert(V * sizeof(T) == 16, "one 16-byte load");
        struct Pack { T v[V]; };
        const vec16_t r = __builtin_nontemporal_load(reinterpret_cast<const vec16_t*>(p));
        const Pack k = __builtin_bit_cast(Pack, r);
#pragma unroll
        for (int j = 0; j < V; ++j) v[j] = k.v[j];
    }
}

constexpr int kValBatch = 8;          // ranks per thread in flight

template <class T, int OP, int V>
__global__ void __launch_bounds__(256) val_partial_kernel(ValArgs A)
{
    __shared__ ValFail vf;
    __shared__ T red[V][256];
    __shared__ double reda[V][256];
    __shared__ uint32_t bad_holder;
    const Geom& g = A.g;
    const uint32_t tid = threadIdx.x;
    const uint32_t s = fdiv(blockIdx.x, A.div_nchunks);
    const uint32_t ch = blockIdx.x - s * A.nchunks;
    const uint32_t c0 = ch * A.chunk;
    const uint32_t c1 = c0 + A.chunk < g.P ? c0 + A.chunk : g.P;
    const uint32_t F = g.f > 0 ? g.f : 1;
    if (tid < 16) {
        uint32_t r = kNoRank, o = 0;
        if (tid < g.f) { r = A.fail_rank[size_t(s) * F + tid]; o = A.fail_round[size_t(s) * F + tid]; }
        vf.rank[tid] = r;
        vf.round[tid] = o;
    }
    if (tid == 0) bad_holder = 0;
    __syncthreads();
    // does the chunk hold a listed rank at all?
    bool chunk_listed = false;
    for (uint32_t q = 0; q < g.f; ++q) chunk_listed = chunk_listed || (vf.rank[q] >= c0 && vf.rank[q] < c1);

    const T* x = reinterpret_cast<const T*>(A.payload + size_t(s) * A.scen_stride_bytes);
    const T* res = reinterpret_cast<const T*>(A.result) + size_t(s) * g.E;
    const T* out = A.out ? reinterpret_cast<const T*>(A.out) + size_t(s) * g.P * g.E : nullptr;
    const uint32_t* hb = A.has_bitmap ? A.has_bitmap + size_t(s) * ((g.P + 31u) / 32u) : nullptr;
    const bool st_ok = A.status[s] == kStOk;
    const bool check_holders = A.kind == 1 && st_ok;
    uint32_t my_bad = 0;

    // a chunk without listed ranks: every process must hold the result; the words of
    // the bitmap are checked here, once (chunks start at multiples of 32 ranks)
    if (check_holders && hb && !chunk_listed && blockIdx.y == 0) {
        const uint32_t w0 = c0 >> 5, nw = (c1 - c0 + 31u) >> 5;
        if (tid < nw) {
            const uint32_t left = c1 - c0 - tid * 32u;
            const uint32_t mask = left >= 32u ? 0xFFFFFFFFu : ((1u << left) - 1u);
            if ((hb[w0 + tid] & mask) != mask) my_bad = 1;
        }
    }

    const uint32_t EV = g.E / uint32_t(V);               // columns of V values
    const uint32_t cols = EV < 256u ? EV : 256u;
    const uint32_t ngr = 256u / cols;
    const uint32_t col = tid % cols, gr = tid / cols;
    {
        // more than 256 columns: the blocks of 256 are workgroups of their own (second grid dimension)
        const uint32_t ev = blockIdx.y * cols + col;
        const uint32_t e = ev * uint32_t(V);
        const bool active = ev < EV && gr < ngr;
        T acc[V];
        double sa[V];
#pragma unroll
        for (int j = 0; j < V; ++j) { acc[j] = T(0); sa[j] = 0.0; }
        if (active) {
            T want[V];
#pragma unroll
            for (int j = 0; j < V; ++j) want[j] = res[e + j];
            for (uint32_t p0 = c0 + gr; p0 < c1; p0 += uint32_t(kValBatch) * ngr) {
                T xv[kValBatch][V], ov[kValBatch][V];
#pragma unroll
                for (int u = 0; u < kValBatch; ++u) {
                    const uint32_t p = p0 + uint32_t(u) * ngr;
                    const size_t at = size_t(p < c1 ? p : c0) * g.E + e;       // past the end: any valid address
                    load_values<T, V>(x + at, xv[u]);
                    if (check_holders && out) load_values<T, V>(out + at, ov[u]);
                }
#pragma unroll
                for (int u = 0; u < kValBatch; ++u) {
                    const uint32_t p = p0 + uint32_t(u) * ngr;
                    if (p >= c1) continue;
                    // 0 never failed, 1 failed before the operation, 2 failed during it
                    uint32_t cls = 0;
                    if (chunk_listed)
                        for (uint32_t q = 0; q < g.f; ++q)
                            if (vf.rank[q] == p) cls = vf.round[q] == 0 ? 1u : 2u;
#pragma unroll
                    for (int j = 0; j < V; ++j) {
                        if (cls == 0) acc[j] = vcomb<T, OP>(acc[j], xv[u][j]);
                        if constexpr (std::is_floating_point<T>::value) {
                            if (cls != 1) sa[j] += fabs(double(xv[u][j]));
                        }
                    }
                    if (check_holders) {
                        bool has = cls == 0, known = cls == 0;
                        if (hb && chunk_listed) {
                            has = ((hb[p >> 5] >> (p & 31u)) & 1u) != 0u;
                            known = true;
                            if ((cls == 0 && !has) || (cls == 1 && has)) my_bad = 1;
                        }
                        if (out && known) {
                            // bitwise comparison, also for floating point: one root, one value
#pragma unroll
                            for (int j = 0; j < V; ++j)
                                if (!same_bits(ov[u][j], has ? want[j] : T(0))) my_bad = 1;
                        }
                    }
                }
            }
        }
        // fold the groups in order
        __syncthreads();
#pragma unroll
        for (int j = 0; j < V; ++j) { red[j][tid] = acc[j]; reda[j][tid] = sa[j]; }
        __syncthreads();
        if (active && gr == 0) {
            for (uint32_t k = 1; k < ngr; ++k) {
#pragma unroll
                for (int j = 0; j < V; ++j) {
                    acc[j] = vcomb<T, OP>(acc[j], red[j][k * cols + col]);
                    sa[j] += reda[j][k * cols + col];
                }
            }
#pragma unroll
            for (int j = 0; j < V; ++j) {
                const size_t o = (size_t(s) * A.nchunks + ch) * g.E + e + uint32_t(j);
                reinterpret_cast<T*>(A.partial)[o * (8 / sizeof(T))] = acc[j];   // one 8-byte slot per value
                A.scale[o] = sa[j];
            }
        }
    }
    if (my_bad) atomicOr(&bad_holder, 1u);
    __syncthreads();
    if (tid == 0 && bad_holder) atomicOr(&A.verdict[s], uint32_t(FTRED_BAD_HOLDER));
}

// group size of the process with virtual rank v (0 = the root), root counted
__device__ __forceinline__ uint32_t vgroup_size(const Geom& g, uint32_t v)
{
    if (v == 0) return g.a > 1 ? g.a : 1u;
    return group_size(g, fdiv(v - 1, g.divW));
}

template <class T, int OP>
__global__ void __launch_bounds__(256) val_final_kernel(ValArgs A)
{
    extern __shared__ __align__(16) unsigned char smem[];
    __shared__ uint32_t s_inop[16], s_fr[16], s_fo[16];
    __shared__ uint32_t s_ninop, s_found, s_expect, s_verdict;
    const Geom& g = A.g;
    const uint32_t tid = threadIdx.x;
    const uint32_t s = blockIdx.x;
    const uint32_t F = g.f > 0 ? g.f : 1;
    T* base = reinterpret_cast<T*>(smem);                               // [E]
    double* scale = reinterpret_cast<double*>(smem + size_t(g.E) * 8u); // [E]
    const T* x = reinterpret_cast<const T*>(A.payload + size_t(s) * A.scen_stride_bytes);
    const T* res = reinterpret_cast<const T*>(A.result) + size_t(s) * g.E;
    const uint32_t nthr = blockDim.x;
    // the failure list goes through LDS: one round trip to memory instead of one per entry
    if (tid < 16) {
        s_fr[tid] = tid < F ? A.fail_rank[size_t(s) * F + tid] : kNoRank;
        s_fo[tid] = tid < F ? A.fail_round[size_t(s) * F + tid] : 0u;
    }
    __syncthreads();
    const uint32_t* fr = s_fr;
    const uint32_t* fo = s_fo;

    // ---- the scenario's failure set: expected status, processes failed during the operation
    if (tid == 0) {
        bool bad = false;
        uint32_t lead = 0, n = 0;
        const uint32_t root = (A.kind == 0 && A.root) ? A.root[s] : 0u;
        bool root_dead = false;
        for (uint32_t q = 0; q < F; ++q) {
            const uint32_t r = fr[q];
            if (r == kNoRank) continue;
            if (q >= g.f || r >= g.P) { bad = true; continue; }
            for (uint32_t q2 = 0; q2 < q; ++q2) bad = bad || fr[q2] == r;
            if (A.kind == 1 && r <= g.f) {
                if (fo[q] != 0) bad = true; else lead |= 1u << r;
            }
            if (fo[q] != 0) s_inop[n++] = r;
            if (A.kind == 0 && r == root && !(fo[q] != 0 && g.Rred < fo[q])) root_dead = true;
        }
        if (A.kind == 0 && root >= g.P) bad = true;
        s_ninop = bad ? 0u : n;
        uint32_t att = 0;
        while ((lead >> att) & 1u) ++att;
        const uint32_t expect = bad ? kStBadFailureSet : (root_dead ? kStRootFailed : kStOk);
        s_expect = expect;
        s_found = 0;
        uint32_t v = 0;
        if (A.status[s] != expect) v |= FTRED_BAD_STATUS;
        if (!bad && A.kind == 1 && A.attempts && A.attempts[s] != att + 1u) v |= FTRED_BAD_STATUS;
        // message counters: between "every listed process sends nothing" and the
        // failure-free counts, per attempt
        if (!bad && A.msgs) {
            const uint32_t natt = A.kind == 1 ? att + 1u : 1u;
            unsigned long long lo_uc = 0, hi_uc = 0, lo_tr = 0, hi_tr = 0;
            for (uint32_t a = 0; a < natt; ++a) {
                const uint32_t rt = A.kind == 1 ? a : root;
                unsigned long long drop_uc = 0, drop_tr = 0;
                for (uint32_t q = 0; q < g.f; ++q) {
                    if (fr[q] == kNoRank) continue;
                    const uint32_t v2 = relabel(fr[q], rt);
                    drop_uc += vgroup_size(g, v2) - 1u;
                    drop_tr += v2 != 0 ? 1u : 0u;
                }
                hi_uc += A.uc_ff; lo_uc += A.uc_ff - drop_uc;
                hi_tr += g.P - 1u; lo_tr += g.P - 1u - drop_tr;
            }
            const unsigned long long* m = A.msgs + size_t(s) * (A.kind == 1 ? 4u : 2u);
            if (m[0] < lo_uc || m[0] > hi_uc || m[1] < lo_tr || m[1] > hi_tr) v |= FTRED_BAD_COUNT;
            if (n == 0 && (m[0] != lo_uc || m[1] != lo_tr)) v |= FTRED_BAD_COUNT;   // exact without in-operation failures
            if (A.kind == 1 && A.status[s] == kStOk) {
                // one broadcast, from a root that is alive
                if (m[2] > g.P - 1u || m[3] > A.uc_ff) v |= FTRED_BAD_COUNT;
                bool none = true;
                for (uint32_t q = 0; q < g.f; ++q) none = none && fr[q] == kNoRank;
                if (none && (m[2] != g.P - 1u || m[3] != A.uc_ff)) v |= FTRED_BAD_COUNT;
            }
        }
        s_verdict = v;          // this pass's findings; only this workgroup touches the scenario's verdict now
    }
    // ---- reduction over the never-failed processes: chunk partials in order
    for (uint32_t e = tid; e < g.E; e += nthr) {
        T acc = T(0);
        double sa = 0.0;
        constexpr uint32_t kAhead = 8;                   // loads in flight; folded in chunk order all the same
        for (uint32_t c0 = 0; c0 < A.nchunks; c0 += kAhead) {
            T pv[kAhead];
            double ps[kAhead];
#pragma unroll
            for (uint32_t u = 0; u < kAhead; ++u) {
                const uint32_t c = c0 + u < A.nchunks ? c0 + u : A.nchunks - 1u;
                const size_t o = (size_t(s) * A.nchunks + c) * g.E + e;
                pv[u] = reinterpret_cast<const T*>(A.partial)[o * (8 / sizeof(T))];
                ps[u] = A.scale[o];
            }
#pragma unroll
            for (uint32_t u = 0; u < kAhead; ++u) {
                if (c0 + u >= A.nchunks) continue;
                acc = vcomb<T, OP>(acc, pv[u]);
                sa += ps[u];
            }
        }
        base[e] = acc;
        scale[e] = sa;
    }
    __syncthreads();
    // ---- one subset of the processes failed during the operation must explain the result
    if (s_expect == kStOk && A.status[s] == kStOk) {
        const uint32_t k = s_ninop;
        const uint32_t nsub = 1u << k;
        uint32_t found = 0;
        if (g.E >= 64u) {
            // many value indices: a wavefront per subset, its lanes side by side over the value indices; a wrong
            // subset is dropped at the first 64 values that do not agree
            const uint32_t lane = tid & 63u, nw = nthr >> 6;
            for (uint32_t sub = tid >> 6; sub < nsub && !found; sub += nw) {
                bool all = true;
                for (uint32_t e0 = 0; e0 < g.E && all; e0 += 64u) {
                    const uint32_t e = e0 + lane;
                    bool ok = true;
                    if (e < g.E) {
                        T cand = base[e];
                        for (uint32_t b = 0; b < k; ++b)
                            if ((sub >> b) & 1u) cand = vcomb<T, OP>(cand, x[size_t(s_inop[b]) * g.E + e]);
                        const T r = res[e];
                        if constexpr (std::is_floating_point<T>::value) ok = fabs(double(r) - double(cand)) <= 1e-12 * scale[e];
                        else ok = r == cand;
                    }
                    all = __all(ok) != 0;
                }
                if (all) found = 1;
            }
        } else
        for (uint32_t sub = tid; sub < nsub && !found; sub += nthr) {
            bool all = true;
            for (uint32_t e = 0; e < g.E && all; ++e) {
                T cand = base[e];
                for (uint32_t b = 0; b < k; ++b)
                    if ((sub >> b) & 1u) cand = vcomb<T, OP>(cand, x[size_t(s_inop[b]) * g.E + e]);
                const T r = res[e];
                if constexpr (std::is_floating_point<T>::value) {
                    // floating point: |r - cand| <= 1e-12 * sum |x|   (false for NaN)
                    all = fabs(double(r) - double(cand)) <= 1e-12 * scale[e];
                } else {
                    all = r == cand;
                }
            }
            if (all) found = 1;
        }
        if (found) atomicOr(&s_found, 1u);
        __syncthreads();
        if (tid == 0 && !s_found) s_verdict |= uint32_t(FTRED_BAD_VALUE);
    }
    __syncthreads();
    if (tid == 0) {
        // pass 1 of this scenario has finished (earlier kernel): its bits are in memory, the verdict is final
        const uint32_t all = A.verdict[s] | s_verdict;
        if (s_verdict != 0u) A.verdict[s] = all;
        if (all != 0u) atomicAdd(A.n_invalid, 1ull);
    }
}

template <class T, int OP>
hipError_t launch_validate(const ValArgs& A, hipStream_t st)
{
    {
        TimedLaunch tl(FTRED_PH_VAL_PARTIAL, st);
        // 16-byte loads where rows, scenarios and base addresses allow them
        constexpr int VMAX = 16 / int(sizeof(T));
        const bool wide = A.g.E % uint32_t(VMAX) == 0 && A.scen_stride_bytes % 16u == 0 &&
                          reinterpret_cast<uintptr_t>(A.payload) % 16u == 0 &&
                          (!A.out || reinterpret_cast<uintptr_t>(A.out) % 16u == 0);
        if (wide) {
            const uint32_t ev = A.g.E / uint32_t(VMAX);
            hipLaunchKernelGGL((val_partial_kernel<T, OP, VMAX>), dim3(A.S * A.nchunks, (ev + 255u) / 256u), dim3(256), 0, st, A);
        } else {
            hipLaunchKernelGGL((val_partial_kernel<T, OP, 1>), dim3(A.S * A.nchunks, (A.g.E + 255u) / 256u), dim3(256), 0, st, A);
        }
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const uint32_t lds = A.g.E * 16u;
    if (lds > 48u * 1024u) {          // more dynamic LDS than a launch gets without asking
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&val_final_kernel<T, OP>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, int(lds));
        if (e != hipSuccess) return e;
    }
    {
        TimedLaunch tl(FTRED_PH_VAL_FINAL, st);
        // one wavefront per scenario unless there are many value indices: the work is a few dependent loads
        hipLaunchKernelGGL((val_final_kernel<T, OP>), dim3(A.S), dim3(A.g.E <= 64u ? 64 : 256), lds, st, A);
    }
    return hipGetLastError();
}

}  // namespace

extern "C" int ftred_validate(const ftred_plan_t* plan, int kind, uint32_t S, const uint32_t* root, const void* payload,
                              uint64_t scen_stride_elems, const uint32_t* fail_rank, const uint32_t* fail_round,
                              const void* result, const uint32_t* has_bitmap, const void* per_process_out,
                              const uint32_t* status, const uint32_t* attempts, const uint64_t* msgs, uint32_t* verdict,
                              uint64_t* n_invalid, void* workspace, uint64_t workspace_bytes, void* hip_stream)
{
    if (!plan) return set_error(FTRED_EINVAL, "ftred_validate: plan is NULL");
    if (kind != 0 && kind != 1) return set_error(FTRED_EINVAL, "ftred_validate: kind must be 0 (reduce) or 1 (allreduce)");
    if (S == 0) return set_error(FTRED_EINVAL, "ftred_validate: S must be >= 1");
    if (!payload || !fail_rank || !fail_round || !result || !status || !verdict)
        return set_error(FTRED_EINVAL, "ftred_validate: payload, failure lists, result, status and verdict are required");
    const Geom& g = plan->g;
    if (scen_stride_elems != 0 && scen_stride_elems < uint64_t(g.P) * g.E)
        return set_error(FTRED_EINVAL, "ftred_validate: scen_stride_elems < P * elems");
    if (!workspace || reinterpret_cast<uintptr_t>(workspace) % 256 != 0)
        return set_error(FTRED_EINVAL, "ftred_validate: workspace must be non-NULL and 256-byte aligned");
    if (workspace_bytes < ws_total(plan, S))
        return set_error(FTRED_EINVAL, "ftred_validate: workspace of %llu bytes, %llu needed",
                         (unsigned long long)workspace_bytes, (unsigned long long)ws_total(plan, S));
    // pass 2 keeps the reduction over the never-failed processes and its scale in LDS: 16 bytes per value index
    if (g.E * 16u > 128u * 1024u)
        return set_error(FTRED_EUNSUPPORTED, "ftred_validate: more than 8192 values per process (%u)", g.E);
    hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);

    ValArgs A;
    memset(&A, 0, sizeof(A));
    A.g = g;
    A.kind = kind;
    A.S = S;
    A.root = kind == 0 ? root : nullptr;
    A.payload = static_cast<const unsigned char*>(payload);
    A.scen_stride_bytes = scen_stride_elems * g.esz;
    A.fail_rank = fail_rank;
    A.fail_round = fail_round;
    A.result = static_cast<const unsigned char*>(result);
    A.has_bitmap = kind == 1 ? has_bitmap : nullptr;
    A.out = kind == 1 ? static_cast<const unsigned char*>(per_process_out) : nullptr;
    A.status = status;
    A.attempts = kind == 1 ? attempts : nullptr;
    A.msgs = reinterpret_cast<const unsigned long long*>(msgs);
    A.verdict = verdict;
    unsigned char* ws = static_cast<unsigned char*>(workspace);
    const uint64_t voff = ws_val_off(plan, S);
    A.chunk = kind == 1 ? plan->val_chunk : plan->val_chunk_reduce;
    A.nchunks = (g.P + A.chunk - 1u) / A.chunk;              // <= val_chunks(plan), which sizes the scratch
    const uint64_t half = uint64_t(S) * A.nchunks * g.E * 8u;
    A.partial = ws + voff;
    A.scale = reinterpret_cast<double*>(ws + voff + half);
    A.n_invalid = reinterpret_cast<unsigned long long*>(ws + ws_ctr_off(plan, S));
    A.div_nchunks = make_fastdiv(A.nchunks);
    A.uc_ff = msgs_uc_ff(g);
    if (uint64_t(S) * A.nchunks >= (uint64_t(1) << 31))
        return set_error(FTRED_EUNSUPPORTED, "ftred_validate: S = %u scenarios need too many workgroups; split the batch", S);

    {
        TimedLaunch tl(FTRED_PH_VAL_FINAL, st);
        hipLaunchKernelGGL(val_init_kernel, dim3((S + 255u) / 256u), dim3(256), 0, st, S, verdict, A.n_invalid);
    }
    HIP_TRY(hipGetLastError());
    hipError_t e;
    if (plan->dtype == FTRED_I64)
        e = plan->op == FTRED_SUM ? launch_validate<unsigned long long, 0>(A, st) : launch_validate<unsigned long long, 1>(A, st);
    else if (plan->dtype == FTRED_U32)
        e = plan->op == FTRED_SUM ? launch_validate<uint32_t, 0>(A, st) : launch_validate<uint32_t, 1>(A, st);
    else
        e = launch_validate<double, 0>(A, st);
    HIP_TRY(e);
    if (n_invalid) {
        unsigned long long host_n = 0;
        HIP_TRY(hipMemcpyAsync(&host_n, A.n_invalid, sizeof(host_n), hipMemcpyDeviceToHost, st));
        HIP_TRY(hipStreamSynchronize(st));
        *n_invalid = host_n;
    }
    return FTRED_OK;
}

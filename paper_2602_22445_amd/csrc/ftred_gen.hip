// Counter-based generation of failure scenarios and integer payloads on the
// device: Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as
// easy as 1, 2, 3", SC'11), written from the published definition.  A draw is
// addressed by counter = (scenario, index, draw, stream) and key = seed, so the
// host can regenerate any scenario alone with the same recipe.
#include <hip/hip_runtime.h>

#include "../../include/ftred.h"
#include "ftred_plan.h"

using namespace ftred;

namespace {

constexpr uint32_t kStreamRoot = 0, kStreamCount = 1, kStreamRank = 2, kStreamTime = 3, kStreamPayload = 4;

struct U4 { uint32_t x, y, z, w; };

__device__ __forceinline__ U4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0, uint32_t k1)
{
    constexpr uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;     // multipliers
    constexpr uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;     // key increments (Weyl sequence)
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t hi0 = __umulhi(M0, c0), lo0 = M0 * c0;
        const uint32_t hi1 = __umulhi(M1, c2), lo1 = M1 * c2;
        const uint32_t n0 = hi1 ^ c1 ^ k0, n1 = lo1, n2 = hi0 ^ c3 ^ k1, n3 = lo0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += W0; k1 += W1;
    }
    return U4{c0, c1, c2, c3};
}

// one thread per scenario
__global__ void gen_failures_kernel(Geom g, uint32_t k0, uint32_t k1, uint32_t S, uint32_t scen0, uint32_t inop_permille,
                                    uint32_t rounds_per_attempt, uint32_t protected_ranks, uint32_t* root_out,
                                    uint32_t* fail_rank, uint32_t* fail_round)
{
    const uint32_t s = blockIdx.x * blockDim.x + threadIdx.x;
    if (s >= S) return;
    const uint32_t sid = scen0 + s;
    const uint32_t F = g.f > 0 ? g.f : 1;
    if (root_out) root_out[s] = __umulhi(philox4x32_10(sid, 0, 0, kStreamRoot, k0, k1).x, g.P);
    const uint32_t count = __umulhi(philox4x32_10(sid, 0, 0, kStreamCount, k0, k1).x, g.f + 1u);
    uint32_t* fr = fail_rank + size_t(s) * F;
    uint32_t* fo = fail_round + size_t(s) * F;
    for (uint32_t i = 0; i < F; ++i) { fr[i] = kNoRank; fo[i] = 0u; }
    // ranks uniform without replacement: redraw on a duplicate
    for (uint32_t i = 0; i < count; ++i) {
        uint32_t draw = 0, r;
        for (;;) {
            r = __umulhi(philox4x32_10(sid, i, draw, kStreamRank, k0, k1).x, g.P);
            bool dup = false;
            for (uint32_t j = 0; j < i; ++j) dup = dup || fr[j] == r;
            if (!dup) break;
            ++draw;
        }
        fr[i] = r;
    }
    if (inop_permille == 0) return;
    // attempts an allreduce trying roots 0,1,2,.. needs: 1 + leading failed candidates
    uint32_t attempts = 1;
    for (uint32_t c = 0; c < protected_ranks; ++c) {
        bool present = false;
        for (uint32_t j = 0; j < count; ++j) present = present || fr[j] == c;
        if (present && attempts == c + 1u) attempts = c + 2u;
    }
    const unsigned long long span = (unsigned long long)attempts * rounds_per_attempt;
    for (uint32_t i = 0; i < count; ++i) {
        const U4 u = philox4x32_10(sid, i, 0, kStreamTime, k0, k1);
        const bool inop = __umulhi(u.x, 1000u) < inop_permille && fr[i] >= protected_ranks;
        fo[i] = inop ? uint32_t(((unsigned long long)u.y * span) >> 32) + 1u : 0u;
    }
}

// one thread per Philox block = two values
template <class T>
__global__ void gen_payload_kernel(uint32_t k0, uint32_t k1, uint32_t scen0, uint32_t n /* values per scenario */,
                                   uint32_t nblk, uint32_t bits, T* payload)
{
    const uint32_t b = blockIdx.x * blockDim.x + threadIdx.x;
    const uint32_t s = blockIdx.y;
    if (b >= nblk) return;
    const U4 u = philox4x32_10(scen0 + s, b, 0, kStreamPayload, k0, k1);
    const unsigned long long mask = bits < 64 ? (1ull << bits) - 1ull : ~0ull;
    const unsigned long long bias = (sizeof(T) == 8 && bits < 64) ? 1ull << (bits - 1) : 0ull;
    const unsigned long long r0 = ((unsigned long long)u.x | ((unsigned long long)u.y << 32)) & mask;
    const unsigned long long r1 = ((unsigned long long)u.z | ((unsigned long long)u.w << 32)) & mask;
    T* dst = payload + size_t(s) * n;
    dst[2u * b] = T(r0 - bias);
    if (2u * b + 1u < n) dst[2u * b + 1u] = T(r1 - bias);
}

}  // namespace

extern "C" int ftred_gen_failures(const ftred_plan_t* plan, uint64_t seed, uint32_t S, uint32_t scen0,
                                  uint32_t inop_permille, uint32_t rounds_per_attempt, uint32_t protected_ranks,
                                  uint32_t* root_out, uint32_t* fail_rank, uint32_t* fail_round, void* hip_stream)
{
    if (!plan || !fail_rank || !fail_round) return set_error(FTRED_EINVAL, "ftred_gen_failures: NULL argument");
    if (S == 0) return set_error(FTRED_EINVAL, "ftred_gen_failures: S must be >= 1");
    if (inop_permille > 1000) return set_error(FTRED_EINVAL, "ftred_gen_failures: inop_permille > 1000");
    if (inop_permille > 0 && rounds_per_attempt == 0)
        return set_error(FTRED_EINVAL, "ftred_gen_failures: rounds_per_attempt must be >= 1 with failures during the operation");
    hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
    {
        TimedLaunch tl(FTRED_PH_GEN, st);
        hipLaunchKernelGGL(gen_failures_kernel, dim3((S + 127u) / 128u), dim3(128), 0, st, plan->g, uint32_t(seed),
                           uint32_t(seed >> 32), S, scen0, inop_permille, rounds_per_attempt, protected_ranks,
                           root_out, fail_rank, fail_round);
    }
    HIP_TRY(hipGetLastError());
    return FTRED_OK;
}

extern "C" int ftred_gen_payload_int(const ftred_plan_t* plan, uint64_t seed, uint32_t S, uint32_t scen0, uint32_t bits,
                                     void* payload, void* hip_stream)
{
    if (!plan || !payload) return set_error(FTRED_EINVAL, "ftred_gen_payload_int: NULL argument");
    if (plan->dtype == FTRED_F64) return set_error(FTRED_EINVAL, "ftred_gen_payload_int: the plan's dtype is not an integer type");
    if (S == 0 || S > 65535) return set_error(FTRED_EINVAL, "ftred_gen_payload_int: S must be 1..65535 per call");
    const uint32_t maxbits = plan->dtype == FTRED_U32 ? 32u : 64u;
    if (bits < 1 || bits > maxbits) return set_error(FTRED_EINVAL, "ftred_gen_payload_int: bits must be 1..%u", maxbits);
    const Geom& g = plan->g;
    const uint32_t n = g.P * g.E;
    const uint32_t nblk = (n + 1u) / 2u;
    hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
    dim3 grid((nblk + 255u) / 256u, S);
    TimedLaunch tl(FTRED_PH_GEN, st);
    if (plan->dtype == FTRED_I64)
        hipLaunchKernelGGL(gen_payload_kernel<long long>, grid, dim3(256), 0, st, uint32_t(seed), uint32_t(seed >> 32),
                           scen0, n, nblk, bits, static_cast<long long*>(payload));
    else
        hipLaunchKernelGGL(gen_payload_kernel<uint32_t>, grid, dim3(256), 0, st, uint32_t(seed), uint32_t(seed >> 32),
                           scen0, n, nblk, bits, static_cast<uint32_t*>(payload));
    HIP_TRY(hipGetLastError());
    return FTRED_OK;
}

// The plan object behind ftred_plan_t, and the error helpers shared by the
// translation units of the library.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ftred_fused.h"
#include "ftred_kernels.h"
#include "ftred_shape.h"
#include "ftred_wave.h"
#include "ftred_wave_general.h"
#include "ftred_wave_unit.h"

struct ftred_plan_s {
    ftred::Geom g;
    int dtype, op;
    uint32_t ntiers;
    ftred::TierDesc tiers[ftred::kMaxTiers];
    uint32_t max_lds;
    uint32_t vroot_off;
    uint64_t ws_scen;           // scratch bytes per scenario (tree tiers)
    uint32_t use_wave;          // the deepest tier runs as one wavefront per subtree
    ftred::WaveLayout wl;
    uint32_t kwalk_given;       // the flags fix the cones a workgroup walks through
    uint32_t use_unit;          // ... with eight lanes per subtree (one value per process)
    uint32_t list_tile;         // ... and the subtrees with listed processes on the LDS-tile list kernel (wide groups)
    ftred::UnitLayout ul;
    uint32_t lift_off, lift_meta_off;   // scratch of the rows the eight-lane kernel folds above its subtrees (ul.lift)
    uint32_t use_fused;         // ... and the levels above it and the root's choice in the same launch
    uint32_t fused_only;        // rows too large for the LDS tiles: no tiers at all, the fused kernel and the register
                                // walk of the listed subtrees do everything
    ftred::FusedLayout fl;
    uint32_t wave_gshift;       // workgroups of the wavefront tier per scenario = 2^wave_gshift
    ftred_plan_s* alt;          // the same plan on LDS tiles only, for runs that carry the lists of failed processes
                                // (set where the tile kernel that runs the listed subtrees then cannot stage a subtree)
    uint32_t use_shape;         // another tree shape than the binary heap: the plain per-depth kernels (ftred_shape.h)
    uint32_t shape_msg_off, shape_meta_off;   // their scratch: the tree messages of every row, one word per row
    uint32_t retry_scratch;     // scratch areas of retry entries (none for the per-depth kernels)
    uint32_t steps[4];          // message steps of one failure-free attempt (ftred_info)
    uint32_t bc_chunk;          // ranks per workgroup in the broadcast kernel
    uint32_t val_chunk;         // ranks per workgroup in the validation kernel (allreduce: inputs and receive buffers)
    uint32_t val_chunk_reduce;  // the same for a reduce (inputs only); >= val_chunk, so the scratch for val_chunk suffices
};

namespace ftred {

// records the message for ftred_last_error() and returns `code`
int set_error(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));

inline uint32_t align_up(uint32_t x, uint32_t a) { return (x + a - 1) / a * a; }

inline uint32_t val_chunks(const ftred_plan_s* p) { return (p->g.P + p->val_chunk - 1) / p->val_chunk; }

// workspace layout: [tree scratch of S scenarios][tree scratch of the retry
// entries: kRetrySlots][validation partials][retry list][fix list][256 bytes
// of counters: +0 invalid scenarios (u64), +8 retry entries (u32), +12, +16 and +20 entries
// of the lists of subtrees (u32)]
inline uint64_t ws_retry_off(const ftred_plan_s* p, uint32_t S) { return uint64_t(S) * p->ws_scen; }
inline uint64_t ws_val_off(const ftred_plan_s* p, uint32_t S)
{
    return (uint64_t(S) + p->retry_scratch) * p->ws_scen;
}
inline uint64_t ws_val_bytes(const ftred_plan_s* p, uint32_t S)
{
    // per (scenario, chunk): E values of the partial reduction and E doubles of |x| sums
    return (uint64_t(S) * val_chunks(p) * (uint64_t(p->g.E) * 8u * 2u) + 255u) / 256u * 256u;
}
inline uint64_t ws_list_off(const ftred_plan_s* p, uint32_t S) { return ws_val_off(p, S) + ws_val_bytes(p, S); }
inline uint64_t ws_list_bytes(const ftred_plan_s* p, uint32_t S)
{
    // at most f failed attempts per scenario, two words each
    return (uint64_t(S) * p->g.f * 8u + 255u) / 256u * 256u;
}
// subtrees the plain register kernel leaves to the list kernels: at most f + 1 per
// scenario or retry entry (room for f + 3), four words each
inline uint64_t ws_fix_off(const ftred_plan_s* p, uint32_t S) { return ws_list_off(p, S) + ws_list_bytes(p, S); }
inline uint64_t ws_fix_bytes(const ftred_plan_s* p, uint32_t S)
{
    // room for the capacity rounded up to whole wavefronts of the register kernel (at most 64 entries each)
    return (((uint64_t(S) + kRetrySlots) * (p->g.f + 3u) + 64u) * 16u + 255u) / 256u * 256u;
}
// two such lists: for the LDS-tile kernel and for the register kernel with failure handling
inline uint64_t ws_wfix_off(const ftred_plan_s* p, uint32_t S) { return ws_fix_off(p, S) + ws_fix_bytes(p, S); }
inline uint64_t ws_ctr_off(const ftred_plan_s* p, uint32_t S) { return ws_wfix_off(p, S) + ws_fix_bytes(p, S); }
inline uint64_t ws_own(const ftred_plan_s* p, uint32_t S) { return ws_ctr_off(p, S) + 256u; }
inline uint64_t ws_total(const ftred_plan_s* p, uint32_t S)
{
    const uint64_t a = ws_own(p, S), b = p->alt ? ws_own(p->alt, S) : 0u;
    return a > b ? a : b;
}

// event-pair timing of kernel launches (ftred_timing_begin / ftred_timing_end)
void tm_mark(int phase, hipStream_t st, bool start);
struct TimedLaunch {
    int phase; hipStream_t st;
    TimedLaunch(int ph, hipStream_t s) : phase(ph), st(s) { tm_mark(phase, st, true); }
    ~TimedLaunch() { tm_mark(phase, st, false); }
};

}  // namespace ftred

#define HIP_TRY(expr)                                                                          \
    do {                                                                                       \
        hipError_t e_ = (expr);                                                                \
        if (e_ != hipSuccess)                                                                  \
            return ftred::set_error(3 /* FTRED_EDEVICE */, "%s: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

// C-ABI of libftred (declared in include/ftred.h): plan, launch logic, and the
// kernels that do not depend on the value type's arithmetic (scenario check,
// index arithmetic for every rank).
#include <hip/hip_runtime.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <mutex>
#include <new>

#include "../../include/ftred.h"
#include "ftred_kernels.h"
#include "ftred_phases.h"
#include "ftred_plan.h"

using namespace ftred;

// ---------------------------------------------------------------------------
// errors

static thread_local char g_err[512] = "";

int ftred::set_error(int code, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

#define fail ftred::set_error

extern "C" const char* ftred_last_error(void) { return g_err; }

#ifndef FTRED_SOURCE_HASH
#define FTRED_SOURCE_HASH "unknown"
#endif
extern "C" const char* ftred_source_hash(void) { return FTRED_SOURCE_HASH; }

// ---------------------------------------------------------------------------
// timing of kernel launches with event pairs

namespace {
struct TimingState {
    bool on = false;
    uint32_t cap = 0, used = 0;
    hipEvent_t* ev = nullptr;      // 2 per record
    int* phase = nullptr;
    bool open = false;
} g_tm;
}  // namespace

void ftred::tm_mark(int phase, hipStream_t st, bool start)
{
    if (!g_tm.on) return;
    if (start) {
        g_tm.open = false;
        if (g_tm.used >= g_tm.cap) return;
        if (hipEventRecord(g_tm.ev[2 * g_tm.used], st) != hipSuccess) return;
        g_tm.phase[g_tm.used] = phase;
        g_tm.open = true;
    } else if (g_tm.open) {
        (void)hipEventRecord(g_tm.ev[2 * g_tm.used + 1], st);
        ++g_tm.used;
        g_tm.open = false;
    }
}

extern "C" int ftred_timing_begin(uint32_t max_records)
{
    if (g_tm.on) return fail(FTRED_EINVAL, "ftred_timing_begin: timing is already on");
    if (max_records == 0 || max_records > (1u << 20)) return fail(FTRED_EINVAL, "ftred_timing_begin: max_records must be 1..2^20");
    g_tm.ev = new (std::nothrow) hipEvent_t[2 * size_t(max_records)];
    g_tm.phase = new (std::nothrow) int[max_records];
    if (!g_tm.ev || !g_tm.phase) return fail(FTRED_ENOMEM, "ftred_timing_begin: out of host memory");
    for (uint32_t i = 0; i < 2 * max_records; ++i) {
        hipError_t e = hipEventCreate(&g_tm.ev[i]);
        if (e != hipSuccess) {
            for (uint32_t k = 0; k < i; ++k) (void)hipEventDestroy(g_tm.ev[k]);
            delete[] g_tm.ev; delete[] g_tm.phase;
            g_tm.ev = nullptr; g_tm.phase = nullptr;
            return fail(FTRED_EDEVICE, "hipEventCreate: %s", hipGetErrorString(e));
        }
    }
    g_tm.cap = max_records;
    g_tm.used = 0;
    g_tm.open = false;
    g_tm.on = true;
    return FTRED_OK;
}

extern "C" int ftred_timing_end(double* ms, uint64_t* launches)
{
    if (!g_tm.on) return fail(FTRED_EINVAL, "ftred_timing_end: timing is not on");
    g_tm.on = false;
    int rc = FTRED_OK;
    if (ms) for (int i = 0; i < FTRED_PH_COUNT; ++i) ms[i] = 0.0;
    if (launches) for (int i = 0; i < FTRED_PH_COUNT; ++i) launches[i] = 0;
    for (uint32_t r = 0; r < g_tm.used; ++r) {
        float t = 0.f;
        hipError_t e = hipEventSynchronize(g_tm.ev[2 * r + 1]);
        if (e == hipSuccess) e = hipEventElapsedTime(&t, g_tm.ev[2 * r], g_tm.ev[2 * r + 1]);
        if (e != hipSuccess) { rc = fail(FTRED_EDEVICE, "ftred_timing_end: %s", hipGetErrorString(e)); break; }
        if (ms) ms[g_tm.phase[r]] += double(t);
        if (launches) launches[g_tm.phase[r]] += 1;
    }
    for (uint32_t i = 0; i < 2 * g_tm.cap; ++i) (void)hipEventDestroy(g_tm.ev[i]);
    delete[] g_tm.ev; delete[] g_tm.phase;
    g_tm.ev = nullptr; g_tm.phase = nullptr;
    g_tm.cap = g_tm.used = 0;
    return rc;
}

// ---------------------------------------------------------------------------
// plan

// Message steps of one failure-free attempt, one port per process (ftred_info.steps_*): in a round every process
// sends at most one up-correction, tree or correction message, so what counts is how many tree messages arrive
// at one process in one round (children of equal height, which send in the same round) and how many children a
// process forwards the broadcast to.  The two sizes a subtree can have are walked position by position.
static void plan_steps(ftred_plan_t* p)
{
    const Geom& g = p->g;
    p->steps[0] = p->steps[1] = p->steps[2] = p->steps[3] = 0;
    if (g.M > (1u << 22)) return;
    p->steps[0] = p->steps[3] = g.f;                 // one message per process and round; a full group exists
    uint32_t fan_in[40] = {0}, fan_out[40] = {0}, root_in[40] = {0};     // by round; D <= 33
    for (uint32_t i = 0; i < g.W; ++i) {
        const uint32_t hi = sh_height_m(g.shape, subtree_size(g, i), 0);
        if (++root_in[hi + 1u] > fan_in[hi + 1u]) fan_in[hi + 1u] = root_in[hi + 1u];
    }
    fan_out[1] = g.W;                                 // the root forwards to its f+1 children
    const uint32_t sizes[2] = {g.M, subtree_size(g, g.W - 1u)};
    for (uint32_t c = 0; c < (sizes[1] != sizes[0] ? 2u : 1u); ++c) {
        const uint32_t m = sizes[c];
        for (uint32_t j = 0; j < m; ++j) {
            uint32_t by_height[40] = {0}, nkids = 0;
            sh_for_children(g, m, j, [&](uint32_t jc) {
                ++nkids;
                const uint32_t r = sh_height_m(g.shape, m, jc) + 1u;       // tree round of this child's message
                if (++by_height[r] > fan_in[r]) fan_in[r] = by_height[r];
            });
            const uint32_t r = sh_depth(g, j) + 1u;                        // broadcast round in which j forwards
            if (nkids > fan_out[r]) fan_out[r] = nkids;
            if (nkids == 0) {
                const uint32_t r0 = sh_height_m(g.shape, m, j) + 1u;       // a sender with no child: one message out
                if (fan_in[r0] == 0) fan_in[r0] = 1;
            }
        }
    }
    for (uint32_t r = 1; r <= g.D && r < 40u; ++r) {
        p->steps[1] += fan_in[r] ? fan_in[r] : 1u;
        p->steps[2] += fan_out[r] ? fan_out[r] : 1u;
    }
}

// Can the deepest tier run on the register walks?  For every width they are built for; beyond the widths of the walk
// with failure handling the listed subtrees go to the LDS-tile list kernel, which stages a whole subtree of the
// walk's height: its rows must fit the prefetch registers and a tile of at most 40 KiB.
static bool wave_usable(const Geom& g)
{
    if (!wave_width_ok(g.W)) return false;
    if (wave_list_width_ok(g.W)) return true;
    const uint32_t per_row = g.RB + 4u + 2u * g.W;
    return kWaveRows <= kStageBytes / g.RB && kWaveRows * per_row <= 40u * 1024u;
}

extern "C" int ftred_plan(ftred_plan_t** out, uint32_t P, uint32_t f, uint32_t elems, int dtype, int op,
                          uint32_t flags)
{
    if (!out) return fail(FTRED_EINVAL, "ftred_plan: out is NULL");
    *out = nullptr;
    if (f > FTRED_MAX_F) return fail(FTRED_EUNSUPPORTED, "ftred_plan: f = %u exceeds %u", f, FTRED_MAX_F);
    if (P < f + 2) return fail(FTRED_EINVAL, "ftred_plan: P = %u < f + 2 = %u (the root needs f+1 children)", P, f + 2);
    if (elems < 1) return fail(FTRED_EINVAL, "ftred_plan: elems must be >= 1");
    if (dtype != FTRED_I64 && dtype != FTRED_U32 && dtype != FTRED_F64)
        return fail(FTRED_EINVAL, "ftred_plan: unknown dtype %d", dtype);
    if (op != FTRED_SUM && op != FTRED_BOR) return fail(FTRED_EINVAL, "ftred_plan: unknown op %d", op);
    if (dtype == FTRED_F64 && op == FTRED_BOR) return fail(FTRED_EINVAL, "ftred_plan: bitwise or needs an integer type");
    const uint32_t esz = dtype == FTRED_U32 ? 4u : 8u;
    if (uint64_t(P) * elems * esz >= (uint64_t(1) << 31))
        return fail(FTRED_EUNSUPPORTED, "ftred_plan: P * elems * size must stay below 2^31 bytes");
    uint32_t budget = 24u * 1024u, kwalk = 3;
    if ((flags & 0xFFu) != 0) {
        if ((flags & 0xFFu) < 4 || (flags & 0xFFu) > 24)
            return fail(FTRED_EINVAL, "ftred_plan: flags bits 0..7 = LDS budget of the deepest tier in KiB, 4..24");
        budget = (flags & 0xFFu) * 1024u;
    }
    const bool kwalk_given = ((flags >> 8) & 0xFu) != 0;
    if (kwalk_given) kwalk = ((flags >> 8) & 0xFu) - 1u;
    if ((flags >> 27) != 0) return fail(FTRED_EINVAL, "ftred_plan: unknown flag bits");
    uint32_t shape = (flags >> 20) & 0x7Fu;
    if (shape == 0) shape = kShapeBinary;
    if (shape > kShapeMaxArity) return fail(FTRED_EINVAL, "ftred_plan: flags bits 20..26 = tree shape: 0 or 2 binary, 1 binomial, k <= 64 children");
    if (((flags >> 17) & 7u) > 5u) return fail(FTRED_EINVAL, "ftred_plan: flags bits 17..19 = 1 + log2(KiB / 4) of a broadcast chunk, 1..5");
    ftred_plan_t* p = new (std::nothrow) ftred_plan_t;
    if (!p) return fail(FTRED_ENOMEM, "ftred_plan: out of host memory");
    memset(p, 0, sizeof(*p));
    p->g = make_geom(P, f, elems, esz, shape);
    p->retry_scratch = kRetrySlots;
    p->dtype = dtype;
    p->op = op;
    const Geom& g = p->g;

    // a row (one up-correction group) must fit the LDS tiles and their prefetch registers; payloads too large for
    // that (the bandwidth regime: kilobytes per process) run on the plain per-depth kernels, which take one thread
    // per (row, value index) and have no such limit
    bool row_too_large = (kStageBytes / g.RB) < 1u || ((56u * 1024u) / (g.RB + 4u + 2u * g.W)) < 3u ||
                         (budget / (g.RB + 4u + 2u * g.W)) < 1u;
    if (!row_too_large) {
        // ... or so few rows fit a tile that the tree would be cut into more tiers than a plan holds
        const uint32_t stage_rows = kStageBytes / g.RB, per_row = g.RB + 4u + 2u * g.W;
        uint32_t c0 = budget / per_row, c1 = (56u * 1024u) / per_row;
        if (c0 > stage_rows) c0 = stage_rows;
        if (c1 > 2u * stage_rows + 1u) c1 = 2u * stage_rows + 1u;
        const uint32_t hc0 = ilog2(c0 + 1u) - 1u, hc1 = ilog2(c1 + 1u) - 2u;
        const bool wave = g.L > uint32_t(kWaveH) && !(flags & 0x1000u) && wave_usable(g);
        const uint32_t h0 = wave ? uint32_t(kWaveH) : (hc0 < g.L ? hc0 : g.L);
        const uint32_t levels = g.L - h0;
        if (1u + (levels + hc1) / (hc1 + 1u) > uint32_t(kMaxTiers)) row_too_large = true;
    }
    bool info_alt = false;
    // ... unless one workgroup can fold a whole scenario, block of value indices by block: that kernel and the
    // register walk of the listed subtrees need no LDS tile of rows at all
    if (shape == kShapeBinary && row_too_large && g.L > uint32_t(kWaveH) && !(flags & 0x11000u) && !((flags >> 13) & 7u) &&
        wave_list_width_ok(g.W) && g.E > 1u && make_fused_layout(g, g.L - uint32_t(kWaveH)).ok) {
        p->fused_only = 1;
        p->use_wave = 1;
        p->use_fused = 1;
        TierDesc& t = p->tiers[0];
        t.dlo = g.L - uint32_t(kWaveH); t.dhi = g.L;
        p->ntiers = 1;
        p->vroot_off = 0;
        uint32_t off = align_up(g.EB, 16);               // [0, EB): the root's value after up-correction
        t.out_off = off;                                 // the top rows of the listed subtrees and their words
        off += align_up((1u << t.dlo) * g.RB, 16);
        t.out_meta_off = off;
        off += align_up((1u << t.dlo) * 4u, 16);
        p->ws_scen = align_up(off, 256);
        p->wl = make_wave_layout(g, t.dlo);
        p->fl = make_fused_layout(g, t.dlo);
    } else
    if (shape != kShapeBinary || row_too_large) {
        // the plain per-depth kernels: no tiers; scratch = the root's value, the tree messages of every row, a word per row
        p->use_shape = 1;
        p->retry_scratch = 0;
        p->vroot_off = 0;
        p->shape_msg_off = align_up(g.EB, 16);
        p->shape_meta_off = p->shape_msg_off + align_up(g.M * g.RB, 16);
        p->ws_scen = align_up(p->shape_meta_off + g.M * 4u, 256);
        if (uint64_t(align_up(g.EB, 16)) + uint64_t(g.M) * g.RB + uint64_t(g.M) * 4u + 512u >= (uint64_t(1) << 32)) {
            delete p;
            return fail(FTRED_EUNSUPPORTED, "ftred_plan: the scratch of one scenario must stay below 4 GiB");
        }
    }
    if (!p->use_shape && !p->fused_only) {
        // tiers of the tree phase, deepest first.  The deepest tier reads the payload
        // and wants many workgroups per CU (small tiles); the upper tiers are small.
        const uint32_t stage_rows = kStageBytes / g.RB;               // rows the prefetch registers hold
        const uint32_t per_row = g.RB + 4u + 2u * g.W;          // values, meta word, lists
        // groups too wide for the register walk with failure handling: the deepest tier's tile serves the list of
        // subtrees with listed processes alone, and must hold one such subtree whatever the budget asked for
        const bool list_tile = g.L > uint32_t(kWaveH) && !(flags & 0x1000u) && !wave_list_width_ok(g.W) &&
                               wave_usable(g);
        if (list_tile && budget < kWaveRows * per_row) budget = kWaveRows * per_row;
        uint32_t cap0 = budget / per_row;
        uint32_t cap1 = (56u * 1024u) / per_row;
        if (cap0 > stage_rows) cap0 = stage_rows;
        if (cap1 > 2u * stage_rows + 1u) cap1 = 2u * stage_rows + 1u;
        if (cap0 < 1 || cap1 < 3) {
            delete p;
            return fail(FTRED_EUNSUPPORTED, "ftred_plan: one up-correction group (%u bytes) does not fit the LDS tile", g.RB);
        }
        const uint32_t hcap0 = ilog2(cap0 + 1u) - 1u;            // 2^(h+1) - 1 <= cap0
        const uint32_t hcap1 = ilog2(cap1 + 1u) - 2u;            // 2^(h+2) - 1 <= cap1
        uint32_t nt = 0;
        // When the lists of failed processes are asked for, the listed subtrees of the register tier run on the
        // LDS-tile list kernel, which must stage a whole subtree of height kWaveH; where it cannot, such runs take
        // a second plan that is on LDS tiles throughout (p->alt, below).
        p->use_wave = (g.L > uint32_t(kWaveH) && !(flags & 0x1000u) && wave_usable(g)) ? 1u : 0u;
        p->list_tile = list_tile ? 1u : 0u;
        info_alt = p->use_wave && ((2u << kWaveH) - 1u) > cap0;
        // one value per process: the kernel of the deepest tier (eight lanes per subtree) also folds the levels up
        // to the common ancestor of the sibling subtrees a wavefront walks, so the tiers above start that much
        // higher.  The lists of failed processes do not travel through those levels: such runs take the second plan.
        uint32_t lift = 0;
        if (p->use_wave && g.E == 1u && !(flags & 0x10000u)) lift = unit_lift(g.L - uint32_t(kWaveH));
        // several values per process: one workgroup folds a whole scenario where the top rows of its subtrees fit the
        // LDS tile, else the part of the tree below one row of depth dp (the smallest dp that fits); the tiers above
        // then start at depth dp - 1.  `skip` = levels between the deepest tier and the tiers above, either way.
        uint32_t fused_dp = kNoRank;
        if (p->use_wave && g.E > 1u && !list_tile && !(flags & 0x10000u) && !((flags >> 13) & 7u)) {
            const uint32_t dl = g.L - uint32_t(kWaveH);
            for (uint32_t dp = 0; dp + 1u <= dl && fused_dp == kNoRank; ++dp)
                if (make_fused_layout(g, dl, dp).ok) fused_dp = dp;
        }
        const uint32_t skip = fused_dp != kNoRank && fused_dp != 0u ? (g.L - uint32_t(kWaveH)) - fused_dp : lift;
        if (skip) info_alt = true;
        {
            uint32_t h0 = hcap0 < g.L ? hcap0 : g.L;
            if (p->use_wave) h0 = uint32_t(kWaveH);
            TierDesc& t = p->tiers[nt++];
            t.dlo = g.L - h0; t.dhi = g.L; t.child_in = 0;
            // the levels above, split evenly over as few tiers as the tile allows: small cones are many workgroups
            // of few threads, which is what these latency-bound launches want
            int d = int(t.dlo) - int(skip) - 1;
            const uint32_t levels = t.dlo - skip, upper = (levels + hcap1) / (hcap1 + 1u);      // tiers above the deepest one
            const uint32_t per = upper ? (levels + upper - 1u) / upper : 0u;             // levels of each but the top one
            while (d >= 0) {
                if (nt == kMaxTiers) {
                    delete p;
                    return fail(FTRED_EUNSUPPORTED, "ftred_plan: the tree needs more than %d tiers at this LDS budget", kMaxTiers);
                }
                uint32_t h = per - 1u < uint32_t(d) ? per - 1u : uint32_t(d);
                TierDesc& u = p->tiers[nt++];
                u.dlo = uint32_t(d) - h; u.dhi = uint32_t(d); u.child_in = 1;
                d = int(u.dlo) - 1;
            }
        }
        p->ntiers = nt;
        p->kwalk_given = kwalk_given ? 1u : 0u;
        uint32_t off = align_up(g.EB, 16);      // [0, EB): the root's value after up-correction
        p->vroot_off = 0;
        for (uint32_t t = 0; t < nt; ++t) {
            TierDesc& td = p->tiers[t];
            const uint32_t h = td.dhi - td.dlo;
            td.is_top = td.dlo == 0 ? 1u : 0u;
            td.lds_rows = ((2u << h) - 1u) + (td.child_in ? (2u << h) : 0u);
            td.lds_bytes = uint32_t(sizeof(FailTab)) + align_up(td.lds_rows * 4u, 16) + align_up(td.lds_rows * g.RB, 16) +
                           align_up(td.lds_rows * g.W * 2u, 16);      // failure table, meta words, rows, lists
            if (td.lds_bytes > p->max_lds) p->max_lds = td.lds_bytes;
            td.kshift = td.dlo < kwalk ? td.dlo : kwalk;
            td.gshift = td.dlo - td.kshift;
            // A small cone is a matter of latency and of instructions every wavefront repeats: no more wavefronts
            // than its widest level has work for, but enough threads for the prefetch registers to hold its rows.
            td.threads = uint32_t(kThreads);
            // (The deepest tier's tile kernel: where the register walks run that tier it serves only the list of
            // subtrees with listed processes, an entry at a time; small entries then want small workgroups, many
            // of them at once.)
            if (t > 0 || p->use_wave) {
                const uint32_t own_bytes = ((2u << h) - 1u) * g.RB, widest = (1u << h) * g.E;
                uint32_t thr = 64;
                while (thr < uint32_t(kThreads) && (thr * kStagePerThread < own_bytes || thr < widest)) thr *= 2u;
                td.threads = thr;
            }
            if (t > 0) {
                td.in_off = p->tiers[t - 1].out_off; td.in_meta_off = p->tiers[t - 1].out_meta_off;
                td.in_mask_off = p->tiers[t - 1].out_mask_off;
            }
            if (t == 1 && skip) {
                // the children of this tier's deepest rows are the rows the kernel of the deepest tier has lifted
                const uint32_t rows = 1u << (p->tiers[0].dlo - skip);
                p->lift_off = off;
                off += align_up(rows * g.RB, 16);
                p->lift_meta_off = off;
                off += align_up(rows * 4u, 16);
                td.in_off = p->lift_off; td.in_meta_off = p->lift_meta_off;
            }
            if (!td.is_top) {
                td.out_off = off;
                off += align_up((1u << td.dlo) * g.RB, 16);
                td.out_meta_off = off;
                off += align_up((1u << td.dlo) * 4u, 16);
                td.out_mask_off = off;
                off += align_up((1u << td.dlo) * g.W * 2u, 16);
            }
        }
        if (p->use_wave) {
            p->wl = make_wave_layout(g, p->tiers[0].dlo);
            const uint32_t most = p->tiers[0].dlo - p->wl.slot_shift;
            if ((flags >> 13) & 7u) p->wl.group_shift = ((flags >> 13) & 7u) - 1u < most ? ((flags >> 13) & 7u) - 1u : most;
            p->wave_gshift = most - p->wl.group_shift;                // one wavefront per workgroup
            p->wl.stage = (p->wl.group_shift > 0 && wave_can_stage(g, p->wl)) ? 1u : 0u;
            p->use_unit = g.E == 1u ? 1u : 0u;
            if (fused_dp != kNoRank) {
                p->fl = make_fused_layout(g, p->tiers[0].dlo, fused_dp);
                p->use_fused = p->fl.ok;
            }
            if (p->use_unit) {
                p->ul = make_unit_layout(p->tiers[0].dlo, g.W);
                p->ul.lift = lift;
                const uint32_t mostu = p->tiers[0].dlo - p->ul.slot_shift;
                if ((flags >> 13) & 7u) p->ul.group_shift = ((flags >> 13) & 7u) - 1u < mostu ? ((flags >> 13) & 7u) - 1u : mostu;
                p->wave_gshift = mostu - p->ul.group_shift;
            }
        }
        p->ws_scen = align_up(off, 256);
    }
    // broadcast / validation chunks: about 32 KiB of payload, a multiple of 32 ranks
    {
        const uint32_t bc_bytes = ((flags >> 17) & 7u) ? (4096u << (((flags >> 17) & 7u) - 1u)) : 32u * 1024u;
        uint32_t c = bc_bytes / g.EB;
        c = c / 32u * 32u;
        if (c < 32u) c = 32u;
        if (c > 8192u) c = 8192u;
        p->bc_chunk = c;
        uint32_t vc = (32u * 1024u) / g.EB / 32u * 32u;
        if (vc < 32u) vc = 32u;
        if (vc > 8192u) vc = 8192u;
        p->val_chunk = vc;
        // the validation of a reduce reads the inputs only: twice the ranks for the same bytes per workgroup
        uint32_t v = (64u * 1024u) / g.EB / 32u * 32u;
        if (v < 32u) v = 32u;
        if (v > 8192u) v = 8192u;
        p->val_chunk_reduce = v;
    }
    plan_steps(p);
    if (info_alt) {
        const int rc = ftred_plan(&p->alt, P, f, elems, dtype, op, (flags & 0xFFFu) | 0x1000u | (flags & ~0x1FFFFu));
        if (rc != FTRED_OK) { delete p; return rc; }
    }
    *out = p;
    return FTRED_OK;
}

extern "C" void ftred_plan_destroy(ftred_plan_t* plan)
{
    if (plan) delete plan->alt;
    delete plan;
}

extern "C" int ftred_plan_info(const ftred_plan_t* plan, ftred_info_t* info)
{
    if (!plan || !info) return fail(FTRED_EINVAL, "ftred_plan_info: NULL argument");
    const Geom& g = plan->g;
    memset(info, 0, sizeof(*info));
    info->P = g.P; info->f = g.f; info->elems = g.E;
    info->dtype = uint32_t(plan->dtype); info->op = uint32_t(plan->op);
    info->groups_full = (g.P - 1) / g.W;
    info->a = g.a;
    info->D = g.D;
    info->rounds_reduce = g.Rred;
    info->rounds_attempt = g.Ratt;
    info->tiers = plan->ntiers;
    info->deep_kernel = plan->use_wave ? (plan->use_unit ? 2u : 1u) : 0u;
    info->fused = plan->use_fused;
    info->shape = g.shape;
    info->steps_uc = plan->steps[0]; info->steps_tree = plan->steps[1];
    info->steps_bcast_tree = plan->steps[2]; info->steps_bcast_corr = plan->steps[3];
    info->msgs_uc_ff = msgs_uc_ff(g);
    info->msgs_tree_ff = g.P - 1;
    info->msgs_bcast_tree_ff = g.P - 1;
    info->msgs_bcast_corr_ff = msgs_uc_ff(g);
    return FTRED_OK;
}

extern "C" uint64_t ftred_workspace_bytes(const ftred_plan_t* plan, uint32_t S)
{
    if (!plan) return 0;
    return ws_total(plan, S);
}

// ---------------------------------------------------------------------------
// index arithmetic of one process, on the host

extern "C" int ftred_partners(const ftred_plan_t* plan, uint32_t root, uint32_t rank, ftred_partners_t* out)
{
    if (!plan || !out) return fail(FTRED_EINVAL, "ftred_partners: NULL argument");
    const Geom& g = plan->g;
    if (root >= g.P || rank >= g.P) return fail(FTRED_EINVAL, "ftred_partners: rank or root >= P");
    memset(out, 0, sizeof(*out));
    PartnerInfo pi;
    partners_of(g, root, rank, pi);
    out->parent = pi.parent;
    out->n_children = pi.n_children;
    for (uint32_t i = 0; i < pi.n_children; ++i) out->children[i] = pi.children[i];
    out->group_size = pi.group_size;
    out->group_pos = pi.group_pos;
    for (uint32_t i = 0; i < pi.group_size; ++i) out->group[i] = pi.group[i];
    out->subtree = pi.subtree;
    out->depth = pi.depth;
    out->height = pi.height;
    out->send_round = pi.send_round;
    return FTRED_OK;
}

__global__ void structure_kernel(Geom g, uint32_t root, uint32_t* parent, uint32_t* subtree, uint32_t* group_id,
                                 uint32_t* group_pos, uint32_t* group_size_out, uint32_t* depth,
                                 uint32_t* send_round)
{
    uint32_t p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= g.P) return;
    PartnerInfo pi;
    partners_of(g, root, p, pi);
    if (parent) parent[p] = pi.parent;
    if (subtree) subtree[p] = pi.subtree;
    if (group_id) group_id[p] = pi.group_id;
    if (group_pos) group_pos[p] = pi.group_pos;
    if (group_size_out) group_size_out[p] = pi.group_size;
    if (depth) depth[p] = pi.depth;
    if (send_round) send_round[p] = pi.send_round;
}

extern "C" int ftred_structure(const ftred_plan_t* plan, uint32_t root, uint32_t* parent, uint32_t* subtree,
                               uint32_t* group_id, uint32_t* group_pos, uint32_t* group_size_out,
                               uint32_t* depth, uint32_t* send_round, void* hip_stream)
{
    if (!plan) return fail(FTRED_EINVAL, "ftred_structure: plan is NULL");
    if (root >= plan->g.P) return fail(FTRED_EINVAL, "ftred_structure: root >= P");
    hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
    const uint32_t grid = (plan->g.P + 255u) / 256u;
    hipLaunchKernelGGL(structure_kernel, dim3(grid), dim3(256), 0, st, plan->g, root, parent, subtree, group_id,
                       group_pos, group_size_out, depth, send_round);
    HIP_TRY(hipGetLastError());
    return FTRED_OK;
}

extern "C" int ftred_detect(const ftred_plan_t* plan, int kind, uint32_t S, const uint32_t* root,
                            const uint32_t* fail_rank, const uint32_t* fail_round, uint32_t* detected, void* hip_stream)
{
    if (!plan) return fail(FTRED_EINVAL, "ftred_detect: plan is NULL");
    if (kind != 0 && kind != 1) return fail(FTRED_EINVAL, "ftred_detect: kind must be 0 (reduce) or 1 (allreduce)");
    if (S == 0) return fail(FTRED_EINVAL, "ftred_detect: S must be >= 1");
    if (!fail_rank || !fail_round || !detected) return fail(FTRED_EINVAL, "ftred_detect: fail_rank, fail_round and detected are required");
    hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
    hipLaunchKernelGGL(detect_kernel, dim3((S + 255u) / 256u), dim3(256), 0, st, plan->g, uint32_t(kind), S,
                       kind == 0 ? root : static_cast<const uint32_t*>(nullptr), fail_rank, fail_round, detected);
    HIP_TRY(hipGetLastError());
    return FTRED_OK;
}

// ---------------------------------------------------------------------------
// launch helpers

static hipError_t dispatch_tier(const ftred_plan_t* p, const RunArgs& A, uint32_t grid, uint32_t lds, hipStream_t st)
{
    if (p->dtype == FTRED_I64) return p->op == FTRED_SUM ? launch_tier_i64_sum(A, grid, lds, st) : launch_tier_i64_bor(A, grid, lds, st);
    if (p->dtype == FTRED_U32) return p->op == FTRED_SUM ? launch_tier_u32_sum(A, grid, lds, st) : launch_tier_u32_bor(A, grid, lds, st);
    return launch_tier_f64_sum(A, grid, lds, st);
}

static hipError_t dispatch_list(const ftred_plan_t* p, const RunArgs& A, uint32_t grid, uint32_t lds, hipStream_t st)
{
    if (p->dtype == FTRED_I64) return p->op == FTRED_SUM ? launch_list_i64_sum(A, grid, lds, st) : launch_list_i64_bor(A, grid, lds, st);
    if (p->dtype == FTRED_U32) return p->op == FTRED_SUM ? launch_list_u32_sum(A, grid, lds, st) : launch_list_u32_bor(A, grid, lds, st);
    return launch_list_f64_sum(A, grid, lds, st);
}

static hipError_t dispatch_wave_list(const ftred_plan_t* p, const RunArgs& A, uint32_t grid, uint32_t lds, hipStream_t st)
{
    if (p->dtype == FTRED_I64) return p->op == FTRED_SUM ? launch_wave_list_i64_sum(A, p->wl, grid, lds, st) : launch_wave_list_i64_bor(A, p->wl, grid, lds, st);
    if (p->dtype == FTRED_U32) return p->op == FTRED_SUM ? launch_wave_list_u32_sum(A, p->wl, grid, lds, st) : launch_wave_list_u32_bor(A, p->wl, grid, lds, st);
    return launch_wave_list_f64_sum(A, p->wl, grid, lds, st);
}

static hipError_t dispatch_fused(const ftred_plan_t* p, const RunArgs& A, uint32_t grid, uint32_t lds, hipStream_t st)
{
    if (p->dtype == FTRED_I64) return p->op == FTRED_SUM ? launch_fused_i64_sum(A, p->fl, grid, lds, st) : launch_fused_i64_bor(A, p->fl, grid, lds, st);
    if (p->dtype == FTRED_U32) return p->op == FTRED_SUM ? launch_fused_u32_sum(A, p->fl, grid, lds, st) : launch_fused_u32_bor(A, p->fl, grid, lds, st);
    return launch_fused_f64_sum(A, p->fl, grid, lds, st);
}

static hipError_t dispatch_wave(const ftred_plan_t* p, const RunArgs& A, uint32_t grid, hipStream_t st)
{
    if (p->use_unit) {
        if (p->dtype == FTRED_I64) return p->op == FTRED_SUM ? launch_unit_i64_sum(A, p->ul, grid, st) : launch_unit_i64_bor(A, p->ul, grid, st);
        if (p->dtype == FTRED_U32) return p->op == FTRED_SUM ? launch_unit_u32_sum(A, p->ul, grid, st) : launch_unit_u32_bor(A, p->ul, grid, st);
        return launch_unit_f64_sum(A, p->ul, grid, st);
    }
    if (p->dtype == FTRED_I64) return p->op == FTRED_SUM ? launch_wave_i64_sum(A, p->wl, grid, st) : launch_wave_i64_bor(A, p->wl, grid, st);
    if (p->dtype == FTRED_U32) return p->op == FTRED_SUM ? launch_wave_u32_sum(A, p->wl, grid, st) : launch_wave_u32_bor(A, p->wl, grid, st);
    return launch_wave_f64_sum(A, p->wl, grid, st);
}

// the subtrees of the deepest tier that the plain register kernel leaves out
static int launch_listed(const ftred_plan_t* plan, const RunArgs& A, uint32_t S, uint32_t extra, uint64_t wgs, hipStream_t st)
{
    if (A.wave_general) {           // every listed subtree is on the register kernel's list
        const uint32_t lds = (1u << plan->wl.slot_shift) * kWaveRows * uint32_t(sizeof(RowInfo));
        HIP_TRY(dispatch_wave_list(plan, A, uint32_t(wgs), lds, st));
    } else {                        // every listed subtree is on the LDS-tile kernel's list
        uint64_t cap = (uint64_t(S) + extra) * (plan->g.f + 3u);
        const uint64_t most = 4096u * (uint64_t(kThreads) / plan->tiers[0].threads);     // workgroups that walk the list
        HIP_TRY(dispatch_list(plan, A, uint32_t(cap < most ? cap : most), plan->tiers[0].lds_bytes, st));
    }
    return FTRED_OK;
}

// all tiers of one tree phase; `extra` = retry entries that ride along as extra scenarios
static int launch_tiers(const ftred_plan_t* plan, RunArgs& A, uint32_t S, uint32_t extra, hipStream_t st)
{
    for (uint32_t t = 0; t < plan->ntiers; ++t) {
        A.tier = t;
        TimedLaunch tl(t == 0 ? FTRED_PH_TREE_DEEP : FTRED_PH_TREE_UPPER, st);
        if (t == 0 && plan->use_wave) {
            // subtrees with listed processes, the short last group or a ragged bottom are listed and run by the
            // list kernels; the plain register kernel runs all the others
            // the lists of failed processes travel through the tile kernel only; so do the listed subtrees of
            // groups the register walk with failure handling is not built for
            A.wave_general = (A.info || plan->list_tile) ? 0u : 1u;
            // room for f + 3 listed subtrees per scenario or retry entry (at most f + 1 occur), 2^slot_shift of
            // them per wavefront
            const uint64_t wgs = ((uint64_t(S) + extra) * (plan->g.f + 3u) + (1u << plan->wl.slot_shift) - 1u) >> plan->wl.slot_shift;
            A.wfix_cap = uint32_t(wgs << plan->wl.slot_shift);
            hipLaunchKernelGGL(fixlist_kernel, dim3((S + extra + 255u) / 256u), dim3(256), 0, st, A);
            HIP_TRY(hipGetLastError());
            if (plan->use_fused && !A.info) {
                // the listed subtrees first: their top rows are in the scratch area when the workgroup that owns
                // the scenario folds all the others and then everything above them, down to the root's choice
                const uint32_t lds = (1u << plan->wl.slot_shift) * kWaveRows * uint32_t(sizeof(RowInfo));
                HIP_TRY(dispatch_wave_list(plan, A, uint32_t(wgs), lds, st));
                if ((((uint64_t(S) + extra) * plan->fl.passes) << plan->fl.dp) >= (uint64_t(1) << 31))
                    return fail(FTRED_EUNSUPPORTED, "S = %u scenarios need too many workgroups; split the batch", S);
                HIP_TRY(dispatch_fused(plan, A, ((S + extra) * plan->fl.passes) << plan->fl.dp,
                                       fused_lds_bytes(plan->g, plan->fl, plan->tiers[0].dlo), st));
                if (plan->fl.dp == 0u) return FTRED_OK;         // the whole tree and the root's choice
                continue;                                        // the tiers above the parts' top rows follow
            }
            // where the plain kernel goes on above its subtrees (A.lift) it needs the listed subtrees' top rows:
            // the list kernel runs first
            if (A.lift) {
                const int rc = launch_listed(plan, A, S, extra, wgs, st);
                if (rc != FTRED_OK) return rc;
            }
            HIP_TRY(dispatch_wave(plan, A, (S + extra) << plan->wave_gshift, st));
            if (!A.lift) {
                const int rc = launch_listed(plan, A, S, extra, wgs, st);
                if (rc != FTRED_OK) return rc;
            }
        } else {
            // Tiers above the deepest one: how many cones a workgroup walks through follows the batch, unless the
            // plan's flags fix it.  About 2^14 workgroups measured best (enough to fill the chip several times,
            // few enough for the failure table and the first loads of a workgroup to be shared by several cones).
            TierDesc& td = A.tiers[t];
            if (t > 0 && !plan->kwalk_given) {
                uint32_t k = 0;
                while (k < 3u && k < td.dlo && ((uint64_t(S) + extra) << (td.dlo - k - 1u)) >= 12288u) ++k;
                td.kshift = k;
                td.gshift = td.dlo - k;
            }
            HIP_TRY(dispatch_tier(plan, A, (S + extra) << td.gshift, plan->tiers[t].lds_bytes, st));
        }
    }
    return FTRED_OK;
}

// The tree phase of the other tree shapes: one launch per depth, deepest first, then the root's choice; the
// messages of attempts whose root had failed (allreduce) are counted from the failure lists.
static int launch_shape(const ftred_plan_t* plan, RunArgs& A, uint32_t S, hipStream_t st)
{
    const Geom& g = plan->g;
    TimedLaunch tl(FTRED_PH_TREE_DEEP, st);
    for (uint32_t d = g.D; d >= 1; --d) {           // the rows of a subtree have depths 1 .. D
        ShapeLevel lv;
        memset(&lv, 0, sizeof(lv));
        lv.depth = d;
        lv.msg_off = plan->shape_msg_off;
        lv.meta_off = plan->shape_meta_off;
        if (g.shape == kShapeBinomial) {
            // depth = 1 + number of one bits of the position: no range; the first such position is 2^(d-1) - 1
            lv.j_lo = d > 32u ? g.M : uint32_t((uint64_t(1) << (d - 1u)) - 1u);
            lv.j_hi = g.M;
            lv.filter = 1;
        } else {
            // level d-1 of a k-ary heap: positions (k^(d-1) - 1) / (k - 1) .. + k^(d-1) - 1
            uint64_t first = 0, count = 1;
            for (uint32_t l = 1; l < d && first < g.M; ++l) { first += count; count *= g.shape; }
            lv.j_lo = first < g.M ? uint32_t(first) : g.M;
            lv.j_hi = first + count < g.M ? uint32_t(first + count) : g.M;
        }
        if (lv.j_lo >= lv.j_hi) continue;
        const uint64_t items = uint64_t(lv.j_hi - lv.j_lo) * g.E;
        lv.blocks_per_scen = uint32_t((items + 255u) / 256u);
        lv.div_bps = make_fastdiv(lv.blocks_per_scen);
        if (uint64_t(S) * lv.blocks_per_scen >= (uint64_t(1) << 31))
            return fail(FTRED_EUNSUPPORTED, "this tree shape: S = %u scenarios need too many workgroups; split the batch", S);
        const uint32_t grid = S * lv.blocks_per_scen;
        hipError_t e;
        if (plan->dtype == FTRED_I64) e = plan->op == FTRED_SUM ? launch_shape_level_i64_sum(A, lv, grid, st) : launch_shape_level_i64_bor(A, lv, grid, st);
        else if (plan->dtype == FTRED_U32) e = plan->op == FTRED_SUM ? launch_shape_level_u32_sum(A, lv, grid, st) : launch_shape_level_u32_bor(A, lv, grid, st);
        else e = launch_shape_level_f64_sum(A, lv, grid, st);
        HIP_TRY(e);
    }
    hipError_t e;
    if (plan->dtype == FTRED_I64) e = plan->op == FTRED_SUM ? launch_shape_root_i64_sum(A, plan->shape_msg_off, plan->shape_meta_off, S, st) : launch_shape_root_i64_bor(A, plan->shape_msg_off, plan->shape_meta_off, S, st);
    else if (plan->dtype == FTRED_U32) e = plan->op == FTRED_SUM ? launch_shape_root_u32_sum(A, plan->shape_msg_off, plan->shape_meta_off, S, st) : launch_shape_root_u32_bor(A, plan->shape_msg_off, plan->shape_meta_off, S, st);
    else e = launch_shape_root_f64_sum(A, plan->shape_msg_off, plan->shape_meta_off, S, st);
    HIP_TRY(e);
    if (A.retry_list && g.f > 0) {
        // at most f failed attempts per scenario
        const uint64_t most = uint64_t(S) * g.f;
        hipLaunchKernelGGL(retry_counts_kernel, dim3(uint32_t((most + 255u) / 256u)), dim3(256), 0, st, A,
                           (unsigned long long)msgs_uc_ff(g), 0u);
        HIP_TRY(hipGetLastError());
    }
    return FTRED_OK;
}

static int check_common(const char* who, const ftred_plan_t* plan, uint32_t S, const void* payload,
                        uint64_t scen_stride_elems, const uint32_t* fail_rank, const uint32_t* fail_round,
                        const void* workspace, uint64_t workspace_bytes)
{
    if (!plan) return fail(FTRED_EINVAL, "%s: plan is NULL", who);
    if (S == 0) return fail(FTRED_EINVAL, "%s: S must be >= 1", who);
    if (!payload || !fail_rank || !fail_round) return fail(FTRED_EINVAL, "%s: payload, fail_rank and fail_round are required", who);
    const Geom& g = plan->g;
    if (scen_stride_elems != 0 && scen_stride_elems < uint64_t(g.P) * g.E)
        return fail(FTRED_EINVAL, "%s: scen_stride_elems %llu < P * elems", who, (unsigned long long)scen_stride_elems);
    if (reinterpret_cast<uintptr_t>(payload) % g.esz != 0) return fail(FTRED_EINVAL, "%s: payload is not aligned to its element size", who);
    if (!workspace) return fail(FTRED_EINVAL, "%s: workspace is NULL", who);
    if (reinterpret_cast<uintptr_t>(workspace) % 256 != 0) return fail(FTRED_EINVAL, "%s: workspace must be 256-byte aligned", who);
    if (workspace_bytes < ftred_workspace_bytes(plan, S))
        return fail(FTRED_EINVAL, "%s: workspace of %llu bytes, %llu needed", who, (unsigned long long)workspace_bytes,
                    (unsigned long long)ftred_workspace_bytes(plan, S));
    for (uint32_t t = 0; t < plan->ntiers; ++t) {
        uint32_t sh = plan->tiers[t].gshift;
        if (t == 0 && plan->use_wave && plan->wave_gshift > sh) sh = plan->wave_gshift;
        if (t > 0) sh = plan->tiers[t].dlo;                       // at most one workgroup per cone
        if (((uint64_t(S) + kRetrySlots) << sh) >= (uint64_t(1) << 31))
            return fail(FTRED_EUNSUPPORTED, "%s: S = %u scenarios need too many workgroups; split the batch", who, S);
    }
    return FTRED_OK;
}

static void fill_run_args(RunArgs& A, const ftred_plan_t* p, uint32_t S, const void* payload, uint64_t scen_stride_elems,
                          const uint32_t* fail_rank, const uint32_t* fail_round, void* workspace)
{
    memset(&A, 0, sizeof(A));
    const Geom& g = p->g;
    A.g = g;
    A.payload = static_cast<const unsigned char*>(payload);
    A.scen_stride_bytes = scen_stride_elems * g.esz;
    A.fail_rank = fail_rank;
    A.fail_round = fail_round;
    A.S = S;
    A.ws = static_cast<unsigned char*>(workspace);
    A.ws_stride = p->ws_scen;
    A.vroot_off = p->vroot_off;
    A.vec16 = (g.EB % 16 == 0 && reinterpret_cast<uintptr_t>(payload) % 16 == 0 && A.scen_stride_bytes % 16 == 0) ? 1u : 0u;
    A.ntiers = p->ntiers;
    for (uint32_t t = 0; t < p->ntiers; ++t) A.tiers[t] = p->tiers[t];
    A.lift = p->use_unit ? p->ul.lift : 0u;
    A.lift_off = p->lift_off;
    A.lift_meta_off = p->lift_meta_off;
    A.fix_list = reinterpret_cast<uint32_t*>(A.ws + ws_fix_off(p, S));
    A.fix_count = reinterpret_cast<uint32_t*>(A.ws + ws_ctr_off(p, S) + 12u);
    A.wfix_list = reinterpret_cast<uint32_t*>(A.ws + ws_wfix_off(p, S));
    A.wfix_count = reinterpret_cast<uint32_t*>(A.ws + ws_ctr_off(p, S) + 16u);
}

// ---------------------------------------------------------------------------
// reduce

// outputs of the richer failure-information schemes (all three may be nullptr)
struct InfoOut {
    uint32_t* count;
    uint32_t* ids;
    uint32_t* child;
    bool any() const { return count || ids || child; }
};

// the outputs start empty: scenarios without a result keep that
static hipError_t clear_info(const Geom& g, uint32_t S, const InfoOut& io, hipStream_t st)
{
    const size_t F = g.f > 0 ? g.f : 1;
    if (io.count) hipLaunchKernelGGL(fill_words_kernel, dim3((S + 255u) / 256u), dim3(256), 0, st, io.count, size_t(S), 0u);
    if (io.ids)
        hipLaunchKernelGGL(fill_words_kernel, dim3(uint32_t((S * F + 255u) / 256u)), dim3(256), 0, st, io.ids, S * F, kNoRank);
    if (io.child)
        hipLaunchKernelGGL(fill_words_kernel, dim3(uint32_t((size_t(S) * g.W + 255u) / 256u)), dim3(256), 0, st, io.child,
                           size_t(S) * g.W, 0u);
    return hipGetLastError();
}

static int run_reduce_impl(const char* who, const ftred_plan_t* plan, uint32_t S, const uint32_t* root,
                           const void* payload, uint64_t scen_stride_elems, const uint32_t* fail_rank,
                           const uint32_t* fail_round, void* result, uint32_t* status, uint64_t* msgs,
                           const InfoOut& io, void* workspace, uint64_t workspace_bytes, void* hip_stream)
{
    int rc = check_common(who, plan, S, payload, scen_stride_elems, fail_rank, fail_round, workspace, workspace_bytes);
    if (rc != FTRED_OK) return rc;
    if (!result || !status) return fail(FTRED_EINVAL, "%s: result and status are required", who);
    if (reinterpret_cast<uintptr_t>(result) % plan->g.esz != 0)
        return fail(FTRED_EINVAL, "%s: result must be aligned to the element size", who);
    hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
    const Geom& g = plan->g;
    if (io.any() && (plan->use_shape || plan->fused_only))
        return fail(FTRED_EUNSUPPORTED, "%s: the lists of failed processes are carried by the default tree shape and by "
                                        "payloads whose rows fit the LDS tiles only", who);
    if (io.any()) HIP_TRY(clear_info(g, S, io, st));

    {
        TimedLaunch tl(FTRED_PH_CHECK, st);
        hipLaunchKernelGGL(zero_words_kernel, dim3(1), dim3(64), 0, st,
                           reinterpret_cast<uint32_t*>(static_cast<unsigned char*>(workspace) + ws_ctr_off(plan, S) + 8u), 4u);
        hipLaunchKernelGGL(prepass_kernel, dim3((S + 255u) / 256u), dim3(256), 0, st, g, 0u, S, root, fail_rank,
                           fail_round, status, static_cast<uint32_t*>(nullptr),
                           reinterpret_cast<unsigned long long*>(msgs), 2u, static_cast<unsigned char*>(result),
                           static_cast<uint32_t*>(nullptr), static_cast<uint32_t*>(nullptr));
    }
    HIP_TRY(hipGetLastError());

    RunArgs A;
    fill_run_args(A, plan, S, payload, scen_stride_elems, fail_rank, fail_round, workspace);
    A.root = root;
    A.status = status;
    A.result = static_cast<unsigned char*>(result);
    A.msgs = reinterpret_cast<unsigned long long*>(msgs);
    A.nmsg = 2;
    A.info = io.any() ? 1u : 0u;
    A.info_count = io.count;
    A.info_ids = io.ids;
    A.info_child = io.child;
    if (plan->use_shape) return launch_shape(plan, A, S, st);
    return launch_tiers(plan, A, S, 0, st);
}

extern "C" int ftred_run_reduce(const ftred_plan_t* plan, uint32_t S, const uint32_t* root, const void* payload,
                                uint64_t scen_stride_elems, const uint32_t* fail_rank, const uint32_t* fail_round,
                                void* result, uint32_t* status, uint64_t* msgs, void* workspace,
                                uint64_t workspace_bytes, void* hip_stream)
{
    return run_reduce_impl("ftred_run_reduce", plan, S, root, payload, scen_stride_elems, fail_rank, fail_round, result,
                           status, msgs, InfoOut{nullptr, nullptr, nullptr}, workspace, workspace_bytes, hip_stream);
}

extern "C" int ftred_run_reduce_info(const ftred_plan_t* plan, uint32_t S, const uint32_t* root, const void* payload,
                                     uint64_t scen_stride_elems, const uint32_t* fail_rank, const uint32_t* fail_round,
                                     void* result, uint32_t* status, uint64_t* msgs, uint32_t* info_count,
                                     uint32_t* info_ids, uint32_t* info_child, void* workspace,
                                     uint64_t workspace_bytes, void* hip_stream)
{
    if (!info_count && !info_ids && !info_child)
        return fail(FTRED_EINVAL, "ftred_run_reduce_info: at least one of info_count, info_ids, info_child is required");
    if (plan && plan->alt) plan = plan->alt;
    return run_reduce_impl("ftred_run_reduce_info", plan, S, root, payload, scen_stride_elems, fail_rank, fail_round,
                           result, status, msgs, InfoOut{info_count, info_ids, info_child}, workspace, workspace_bytes,
                           hip_stream);
}

// ---------------------------------------------------------------------------
// allreduce

static int run_allreduce_impl(const char* who, const ftred_plan_t* plan, uint32_t S, const void* payload,
                              uint64_t scen_stride_elems, const uint32_t* fail_rank, const uint32_t* fail_round,
                              void* result, uint32_t* has_bitmap, void* per_process_out, uint32_t* status,
                              uint32_t* attempts, uint64_t* msgs, const InfoOut& io, void* workspace,
                              uint64_t workspace_bytes, void* hip_stream)
{
    int rc = check_common(who, plan, S, payload, scen_stride_elems, fail_rank, fail_round, workspace, workspace_bytes);
    if (rc != FTRED_OK) return rc;
    if (!result || !status || !attempts) return fail(FTRED_EINVAL, "%s: result, status and attempts are required", who);
    if (reinterpret_cast<uintptr_t>(result) % plan->g.esz != 0 || reinterpret_cast<uintptr_t>(per_process_out) % plan->g.esz != 0)
        return fail(FTRED_EINVAL, "%s: result and per_process_out must be aligned to the element size", who);
    hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
    const Geom& g = plan->g;
    if (io.any() && (plan->use_shape || plan->fused_only))
        return fail(FTRED_EUNSUPPORTED, "%s: the lists of failed processes are carried by the default tree shape and by "
                                        "payloads whose rows fit the LDS tiles only", who);
    if (io.any()) HIP_TRY(clear_info(g, S, io, st));

    unsigned char* wsb = static_cast<unsigned char*>(workspace);
    uint32_t* retry_list = reinterpret_cast<uint32_t*>(wsb + ws_list_off(plan, S));
    uint32_t* retry_count = reinterpret_cast<uint32_t*>(wsb + ws_ctr_off(plan, S) + 8u);
    {
        TimedLaunch tl(FTRED_PH_CHECK, st);
        hipLaunchKernelGGL(zero_words_kernel, dim3(1), dim3(64), 0, st, retry_count, 4u);     // and the counts of the two lists of subtrees
        hipLaunchKernelGGL(prepass_kernel, dim3((S + 255u) / 256u), dim3(256), 0, st, g, 1u, S,
                           static_cast<const uint32_t*>(nullptr), fail_rank, fail_round, status, attempts,
                           reinterpret_cast<unsigned long long*>(msgs), 4u, static_cast<unsigned char*>(result),
                           retry_list, retry_count);
    }
    HIP_TRY(hipGetLastError());

    RunArgs A;
    fill_run_args(A, plan, S, payload, scen_stride_elems, fail_rank, fail_round, workspace);
    A.attempts = attempts;
    A.status = status;
    A.result = static_cast<unsigned char*>(result);
    A.msgs = reinterpret_cast<unsigned long long*>(msgs);
    A.nmsg = 4;
    A.info = io.any() ? 1u : 0u;
    A.info_count = io.count;
    A.info_ids = io.ids;
    A.info_child = io.child;
    const uint32_t slots = g.f > 0 ? kRetrySlots : 0u;
    A.retry_list = retry_list;
    A.retry_count = retry_count;
    A.retry_slots = slots;
    A.retry_ws = wsb + ws_retry_off(plan, S);

    // attempts whose root had failed beforehand run as extra "scenarios" of the tier launches
    if (plan->use_shape) {
        rc = launch_shape(plan, A, S, st);
    } else {
        if (g.f > 0) {
            // beyond kRetrySlots of them (unusual) nothing is simulated: their messages are counted from the failure lists
            TimedLaunch tl(FTRED_PH_RETRY, st);
            const uint64_t most = uint64_t(S) * g.f;        // at most f failed attempts per scenario
            if (most > slots) {
                hipLaunchKernelGGL(retry_counts_kernel, dim3(uint32_t((most - slots + 255u) / 256u)), dim3(256), 0, st, A,
                                   (unsigned long long)msgs_uc_ff(g), slots);
                HIP_TRY(hipGetLastError());
            }
        }
        rc = launch_tiers(plan, A, S, slots, st);
    }
    if (rc != FTRED_OK) return rc;
    // broadcast down the tree and correction rounds
    BcastArgs B;
    memset(&B, 0, sizeof(B));
    B.g = g;
    B.S = S;
    B.attempts = attempts;
    B.status = status;
    B.fail_rank = fail_rank;
    B.fail_round = fail_round;
    B.result = static_cast<const unsigned char*>(result);
    B.has_bitmap = has_bitmap;
    B.out = static_cast<unsigned char*>(per_process_out);
    B.msgs = reinterpret_cast<unsigned long long*>(msgs);
    B.chunk = plan->bc_chunk;
    B.nchunks = (g.P + plan->bc_chunk - 1) / plan->bc_chunk;
    B.div_nchunks = make_fastdiv(B.nchunks);
    B.vec16 = (g.EB % 16 == 0 && reinterpret_cast<uintptr_t>(result) % 16 == 0 &&
               (!per_process_out || reinterpret_cast<uintptr_t>(per_process_out) % 16 == 0)) ? 1u : 0u;
    // values of 4 or 8 bytes: 4 or 2 receive buffers per 16-byte store (a chunk starts at a multiple of 32 ranks)
    B.small16 = ((g.EB == 4 || g.EB == 8) && per_process_out && reinterpret_cast<uintptr_t>(per_process_out) % 16 == 0 &&
                 (uint64_t(g.P) * g.EB) % 16 == 0) ? 1u : 0u;
    if (uint64_t(S) * B.nchunks >= (uint64_t(1) << 31))
        return fail(FTRED_EUNSUPPORTED, "ftred_run_allreduce: S = %u scenarios need too many workgroups; split the batch", S);
    // the kernel's other instantiation: values that are no multiple of 16 bytes get 16-byte stores where every
    // scenario's buffers start on one, and chunks of many groups (few bytes per process) take their holders and
    // counts from the chunk's place in the tree where no listed process touches them
    B.any16 = (!B.small16 && g.EB % 16 != 0 && g.EB <= 4096u && per_process_out &&
               reinterpret_cast<uintptr_t>(per_process_out) % 16 == 0 && (uint64_t(g.P) * g.EB) % 16 == 0) ? 1u : 0u;
    const bool alt = B.any16 || plan->bc_chunk / g.W >= 256u;
    const uint32_t lds = bcast_lds_bytes(B);
    {
        TimedLaunch tl(FTRED_PH_BCAST, st);
        if (g.shape == kShapeBinary) {
            if (alt) hipLaunchKernelGGL((bcast_kernel<true, true>), dim3(S * B.nchunks), dim3(kThreads), lds, st, B);
            else hipLaunchKernelGGL((bcast_kernel<true, false>), dim3(S * B.nchunks), dim3(kThreads), lds, st, B);
        } else {
            if (alt) hipLaunchKernelGGL((bcast_kernel<false, true>), dim3(S * B.nchunks), dim3(kThreads), lds, st, B);
            else hipLaunchKernelGGL((bcast_kernel<false, false>), dim3(S * B.nchunks), dim3(kThreads), lds, st, B);
        }
    }
    HIP_TRY(hipGetLastError());
    return FTRED_OK;
}

extern "C" int ftred_run_allreduce(const ftred_plan_t* plan, uint32_t S, const void* payload, uint64_t scen_stride_elems,
                                   const uint32_t* fail_rank, const uint32_t* fail_round, void* result,
                                   uint32_t* has_bitmap, void* per_process_out, uint32_t* status, uint32_t* attempts,
                                   uint64_t* msgs, void* workspace, uint64_t workspace_bytes, void* hip_stream)
{
    return run_allreduce_impl("ftred_run_allreduce", plan, S, payload, scen_stride_elems, fail_rank, fail_round, result,
                              has_bitmap, per_process_out, status, attempts, msgs, InfoOut{nullptr, nullptr, nullptr},
                              workspace, workspace_bytes, hip_stream);
}

extern "C" int ftred_run_allreduce_info(const ftred_plan_t* plan, uint32_t S, const void* payload,
                                        uint64_t scen_stride_elems, const uint32_t* fail_rank,
                                        const uint32_t* fail_round, void* result, uint32_t* has_bitmap,
                                        void* per_process_out, uint32_t* status, uint32_t* attempts, uint64_t* msgs,
                                        uint32_t* info_count, uint32_t* info_ids, uint32_t* info_child, void* workspace,
                                        uint64_t workspace_bytes, void* hip_stream)
{
    if (!info_count && !info_ids && !info_child)
        return fail(FTRED_EINVAL, "ftred_run_allreduce_info: at least one of info_count, info_ids, info_child is required");
    if (plan && plan->alt) plan = plan->alt;
    return run_allreduce_impl("ftred_run_allreduce_info", plan, S, payload, scen_stride_elems, fail_rank, fail_round,
                              result, has_bitmap, per_process_out, status, attempts, msgs,
                              InfoOut{info_count, info_ids, info_child}, workspace, workspace_bytes, hip_stream);
}

// ---------------------------------------------------------------------------
// allreduce for callers that cannot allocate: the workspace is a fixed array in
// device memory that belongs to the library

static __device__ __align__(256) unsigned char scratch[FTRED_NOALLOC_WORKSPACE_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
unsigned char* g_scratch_ptr[kMaxDevices];     // the array's address on each device, once known
}  // namespace

// The address of `scratch` on the current device.  Every device holds its own copy of the array at its
// own address; the name itself is only a host-side handle, never a pointer a kernel could use.
static int scratch_of_current_device(unsigned char** out)
{
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(FTRED_EUNSUPPORTED, "ftred_run_allreduce_noalloc: device %d not supported", dev);
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return fail(FTRED_EDEVICE, "ftred_run_allreduce_noalloc: the workspace array has no device address");
        g_scratch_ptr[dev] = static_cast<unsigned char*>(p);
    }
    *out = g_scratch_ptr[dev];
    return FTRED_OK;
}

extern "C" int ftred_run_allreduce_noalloc(const ftred_plan_t* plan, uint32_t S, const void* payload,
                                           uint64_t scen_stride_elems, const uint32_t* fail_rank,
                                           const uint32_t* fail_round, void* result, uint32_t* has_bitmap,
                                           void* per_process_out, uint32_t* status, uint32_t* attempts, uint64_t* msgs,
                                           void* hip_stream)
{
    if (!plan) return fail(FTRED_EINVAL, "ftred_run_allreduce_noalloc: plan is NULL");
    const uint64_t need = ftred_workspace_bytes(plan, S);
    if (need > uint64_t(FTRED_NOALLOC_WORKSPACE_BYTES))
        return fail(FTRED_EUNSUPPORTED,
                    "ftred_run_allreduce_noalloc: S = %u scenarios of this plan need %llu bytes of workspace, the "
                    "library's fixed array holds %llu; use fewer scenarios per call or ftred_run_allreduce",
                    S, (unsigned long long)need, (unsigned long long)FTRED_NOALLOC_WORKSPACE_BYTES);
    unsigned char* ws = nullptr;
    const int rc = scratch_of_current_device(&ws);
    if (rc != FTRED_OK) return rc;
    // Nothing in the workspace has to survive from call to call, and what must start at zero (the counters of the
    // retry entries and of the lists of subtrees) is cleared by the run itself, by a kernel on the caller's stream.
    return run_allreduce_impl("ftred_run_allreduce_noalloc", plan, S, payload, scen_stride_elems, fail_rank, fail_round,
                              result, has_bitmap, per_process_out, status, attempts, msgs,
                              InfoOut{nullptr, nullptr, nullptr}, ws, uint64_t(FTRED_NOALLOC_WORKSPACE_BYTES), hip_stream);
}

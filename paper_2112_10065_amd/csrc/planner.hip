// Kernel choice for one pass of one layer: enumerate the tile variants and reduction splits that
// the shape allows, price each with a small analytic model calibrated on MI355X measurements,
// take the cheapest.  Host code only.  The model:
//
//   blocks       = tiles * splits               concurrent = 256 CUs * blocks_per_CU(variant)
//   t_block      = t0(variant) + steps_per_split * t_step(variant) * share
//                  (share < 1 when fewer blocks than the variant could co-run share a CU)
//   t            = launch + waves(blocks / concurrent) * t_block + t_reduce(splits)
//   t_reduce     = second kernel that sums the fp32 partials: launch + (splits + 1) * out bytes / BW
#include "dp_kernels.h"
#include <cmath>

namespace {

struct Candidate {
    int code;        // override code understood by fast_plan / dma_plan (100.., 200.., 300..)
    int bpc;         // blocks that fit on one CU (LDS / registers)
    float t_step;    // microseconds per reduction step and block on a fully shared CU
    float t0;        // microseconds of prologue + epilogue per block
    int kg = 1;      // reduction groups inside a block: each group walks 1/kg of the block's steps
};

// forward / backward-data candidates
const Candidate kPix[] = {
    {230, 1, 1.30f, 9.0f},   // 256x256x64, 4 waves, 3x3 stride 1 with the pixel strip shared by the three taps of a filter row
    {231, 1, 0.70f, 7.0f},   // the same with 128 pixel rows per tile and three weight stages
    {232, 1, 0.70f, 7.0f},   // the same with 128 output channels per tile (layers with 128 of them)
    {233, 1, 1.15f, 9.0f},   // the same with 224 pixel rows per tile (four waves side by side over the channels)
    {208, 1, 1.55f, 8.0f},   // 256x256x64, 8 waves, direct-to-LDS
    {200, 2, 1.08f, 5.0f},   // 128x128x64 direct-to-LDS
    {204, 3, 0.85f, 4.5f},   // 64x128x64
    {206, 3, 0.85f, 4.5f},   // 128x64x64
    {207, 3, 0.62f, 4.0f},   // 64x64x64
    {201, 4, 1.08f, 4.5f},   // direct-to-LDS with reduction step 32 (channels % 32 only)
    {205, 4, 0.85f, 4.0f},
    {213, 3, 1.30f, 4.5f},
    {210, 1, 1.15f, 6.0f},   // 128x256x64, 8 waves
    {212, 2, 1.30f, 4.5f},   // 64x256x64
    {221, 1, 0.70f, 4.0f},   // reduction step 128 (channels % 128 only): fewer, longer steps for small grids
    {225, 1, 0.70f, 4.0f},
    {222, 1, 1.10f, 4.5f},
    {224, 1, 1.10f, 4.5f},
    {223, 1, 1.90f, 5.0f},
    {226, 1, 0.62f, 5.0f, 4},   // 64x64x64 with 4 / 2 reduction groups per block (no partials in memory)
    {227, 2, 0.62f, 4.5f, 2},
    {228, 1, 0.85f, 5.0f, 2},
    {229, 1, 0.85f, 5.0f, 2},
    {400, 2, 0.75f, 5.5f},   // input patch resident in LDS: 64 x 256 tile (64 reduction channels per tap, stride 1)
    {401, 2, 1.20f, 6.0f},   // same, 128 x 256
    {402, 2, 0.75f, 5.5f},
    {403, 2, 0.72f, 5.5f},
    {404, 1, 0.50f, 0.8f},   // 3x3 only: persistent blocks, weights in registers
    {100, 2, 1.40f, 5.0f},   // register-staged fallbacks (also reduction step 32)
    {101, 3, 1.05f, 4.5f},
    {102, 3, 1.05f, 4.5f},
    {103, 4, 0.75f, 4.0f},
};
// backward-filter candidates (reduction step 32 unless noted)
const Candidate kWg[] = {
    {300, 4, 1.00f, 4.0f},   // 128x128x32 direct-to-LDS
    {303, 4, 0.70f, 3.5f},   // 64x128x32
    {304, 4, 0.70f, 3.5f},   // 128x64x32
    {305, 5, 0.62f, 3.5f},   // 64x64x32
    {308, 3, 1.45f, 4.0f},   // 64x256x32 (few output channels: widest tap tile)
    {306, 3, 0.93f, 4.0f},   // 64x128x64
    {301, 2, 1.75f, 4.5f},   // 128x128x64
    {307, 2, 1.60f, 5.0f},   // 256x128x32, 8 waves
    {314, 2, 1.65f, 5.0f},   // 128x256x32, 8 waves
    {312, 1, 2.90f, 7.0f},   // 256x256x64, 8 waves
    {316, 1, 1.60f, 9.0f},   // 3x3 stride 1: 256 x (3 taps x 64 channels), x strip shared by the taps, padded pixel slots
    {410, 1, 0.13f, 6.0f},   // input patch in LDS, persistent blocks (64 input channels, stride 1); a step = 16 pixels
    {411, 1, 0.10f, 6.0f},   // the same for 3x3 filters with all nine taps in one wave (four waves per block)
    {100, 3, 1.30f, 4.0f},
    {101, 3, 1.00f, 3.5f},
    {102, 3, 1.00f, 3.5f},
    {103, 4, 0.80f, 3.0f},
};
const int kSplits[] = {1, 2, 3, 4, 5, 6, 8, 10, 12, 16, 20, 24, 32, 48, 64, 96, 128, 192, 256};

bool family_plan(const ConvGeom &g, int pass, int code, int splits, GemmPlan *pl)
{
    pl->halo = false;
    pl->wstrip = false;
    if (code >= 400) return halo_plan(g, pass, code, splits, pl);
    if (code >= 200) return dma_plan(g, pass, code, splits, pl);
    return fast_plan(g, pass, code, splits, pl);
}

double price(const ConvGeom &g, int pass, const Candidate &c, const GemmPlan &pl)
{
    const double blocks = (double)pl.tilesA * pl.tilesB * pl.splits;
    const double conc = 256.0 * c.bpc;
    double share = 1.0, waves;
    if (blocks <= conc) {
        const double r = std::ceil(blocks / 256.0);
        share = 0.45 + 0.55 * r / c.bpc;
        waves = 1.0;
    } else {
        const double w = blocks / conc;
        waves = w >= 4.0 ? w : 0.5 * (w + std::ceil(w));
    }
    // a step of reduction length 32 costs about half of a 64 step for the pixel passes
    double t_step = c.t_step;
    if (pass != PASS_WGRAD && pl.BK == 32) t_step *= 0.6;
    const double t_block = c.t0 + (pl.steps_per_split + c.kg - 1) / c.kg * t_step * share;
    double t = 3.0 + waves * t_block;
    if (pl.splits > 1) {
        double out_elems = pass == PASS_FWD ? (double)g.N * g.Ho * g.Wo * g.K
                         : pass == PASS_DGRAD ? (double)g.N * g.H * g.W * g.C
                                              : (double)g.K * g.R * g.S * g.C;
        t += 3.0 + (pl.splits + 1.0) * out_elems * 4.0 / 4.0e6;   // ~4 TB/s for the partial traffic
    }
    return t;
}

}  // namespace

// Eligible fast-path plans of a pass, cheapest first by the model, at most two split counts per tile
// variant; returns how many were written (0: the shape has no fast-path plan).
int auto_plan_list(const ConvGeom &g, int pass, int force_splits, GemmPlan *out, int max_out, int restr)
{
    struct Priced { double t; GemmPlan pl; int code; };
    Priced all[512];
    int n = 0;
    // dense-layer-like shapes (a handful of pixel rows): the pass streams the weight matrix once and
    // is bound by HBM; the smallest tile with about two blocks per CU does that best
    if (pass != PASS_WGRAD && force_splits <= 0) {
        const long long rowsB = pass == PASS_FWD ? (long long)g.N * g.Ho * g.Wo : (long long)g.N * g.H * g.W;
        if (rowsB <= 64) {
            for (int code : {207, 103}) {
                GemmPlan one;
                if (!family_plan(g, pass, code, 1, &one)) continue;
                const long long tiles = (long long)one.tilesA * one.tilesB;
                int splits = (int)((512 + tiles - 1) / tiles), max_splits = one.steps_total / 8;
                if (max_splits < 1) max_splits = 1;
                if (splits > max_splits) splits = max_splits;
                if (family_plan(g, pass, code, splits, &all[n].pl)) { all[n].t = 0.0; all[n].code = code; ++n; break; }
            }
        }
    }
    const Candidate *cands = pass == PASS_WGRAD ? kWg : kPix;
    const int ncand = pass == PASS_WGRAD ? (int)(sizeof(kWg) / sizeof(kWg[0])) : (int)(sizeof(kPix) / sizeof(kPix[0]));
    for (int ci = 0; ci < ncand; ++ci) {
        if (pass != PASS_WGRAD && cands[ci].code >= 400 && (restr & 1)) continue;   // the input-patch kernels store bf16 only
        if (pass == PASS_DGRAD && cands[ci].code >= 230 && cands[ci].code <= 233 && (restr & 1)) continue;   // bf16 staged epilogue only
        int last_splits = -1;
        for (int s : kSplits) {
            if (force_splits > 0 && s != kSplits[0]) break;
            // backward-filter blocks of one split share their inputs through one XCD's L2 only if the
            // split count is a multiple of the 8 XCDs
            if (pass == PASS_WGRAD && force_splits <= 0 && s > 8 && (s % 8) != 0) continue;
            GemmPlan cand;
            if (!family_plan(g, pass, cands[ci].code, force_splits > 0 ? force_splits : s, &cand)) break;
            // reduction step 32 only where 64 does not divide the channel count
            if (pass != PASS_WGRAD && cand.BK == 32 && ((pass == PASS_FWD ? g.C : g.K) % 64) == 0) break;
            if (cand.splits == last_splits) continue;   // the request was clamped to the same plan
            // pixel-strip kernels on a grid of few blocks: each block streams its weights alone, which times well on a warm
            // cache (the measured choice) and badly inside a step
            // (restr bit 2: the caller measures with cold caches and can judge these grids itself)
            if (!(restr & 4) && cands[ci].code >= 230 && cands[ci].code <= 233 && (long long)cand.tilesA * cand.tilesB * cand.splits < 160) continue;
            last_splits = cand.splits;
            if (force_splits <= 0 && cand.splits > 1 && cand.steps_per_split < 4) break;
            if (n < 512) { all[n].t = price(g, pass, cands[ci], cand); all[n].pl = cand; all[n].code = cands[ci].code; ++n; }
        }
    }
    // selection sort of the few that are wanted; per tile variant only its two cheapest splits
    int written = 0;
    int used_code[64], used_cnt[64], nused = 0;
    double t_first = -1.0;   // the model's best time; plans it puts beyond 1.6x of that are not worth a measurement
    while (written < max_out) {
        int best = -1;
        for (int i = 0; i < n; ++i) {
            if (all[i].t < 0.0) continue;
            if (best < 0 || all[i].t < all[best].t) best = i;
        }
        if (best < 0) break;
        if (all[best].t > 0.0) {
            if (t_first < 0.0) t_first = all[best].t;
            else if (all[best].t > ((restr & 4) ? 2.0 : 1.6) * t_first) break;
        }
        int u = 0;
        while (u < nused && used_code[u] != all[best].code) ++u;
        if (u == nused && nused < 64) { used_code[nused] = all[best].code; used_cnt[nused] = 0; ++nused; }
        if (u < 64 && used_cnt[u] < 2) { out[written++] = all[best].pl; ++used_cnt[u]; }
        all[best].t = -1.0;
    }
    return written;
}

// Fills *pl with the cheapest eligible fast-path plan; false if the shape has none.
bool auto_plan(const ConvGeom &g, int pass, int force_splits, GemmPlan *pl, int restr)
{
    return auto_plan_list(g, pass, force_splits, pl, 1, restr) == 1;
}

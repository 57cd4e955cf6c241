// Host side of the kernel launch: the plan (which configuration, which grid) and the dispatch
// to the per-configuration launchers compiled from spmm_launch_cfg.hip.
#include <hip/hip_runtime.h>

#include "spmm_internal.h"

namespace spmm {

#define SPMM_DECLARE_CFG(name) \
    void name(spmm_out_t, int postop, unsigned grid_x, unsigned grid_y, unsigned block, void* stream, const KernelArgs&)
SPMM_DECLARE_CFG(launch_cfg_128_16_4);
SPMM_DECLARE_CFG(launch_cfg_128_16_5);
SPMM_DECLARE_CFG(launch_cfg_128_16_6);
SPMM_DECLARE_CFG(launch_cfg_128_8_4);
SPMM_DECLARE_CFG(launch_cfg_128_8_6);
SPMM_DECLARE_CFG(launch_cfg_128_8_8);
SPMM_DECLARE_CFG(launch_cfg_96_16_4);
SPMM_DECLARE_CFG(launch_cfg_96_16_5);
SPMM_DECLARE_CFG(launch_cfg_96_16_6);
SPMM_DECLARE_CFG(launch_cfg_fed_128_12_4);
SPMM_DECLARE_CFG(launch_cfg_fed_128_12_6);
SPMM_DECLARE_CFG(launch_cfg_fed_128_8_4);
SPMM_DECLARE_CFG(launch_cfg_fed_128_8_6);
SPMM_DECLARE_CFG(launch_cfg_fed_128_8_8);
SPMM_DECLARE_CFG(launch_cfg_fed_96_12_4);
SPMM_DECLARE_CFG(launch_cfg_fed_96_12_6);
SPMM_DECLARE_CFG(launch_cfg_fed_64_12_4);
SPMM_DECLARE_CFG(launch_cfg_fed_64_12_6);
SPMM_DECLARE_CFG(launch_cfg_simple_1);
SPMM_DECLARE_CFG(launch_cfg_simple_2);
SPMM_DECLARE_CFG(launch_cfg_simple32_1);
SPMM_DECLARE_CFG(launch_cfg_simple16_1);
SPMM_DECLARE_CFG(launch_cfg_slab16);
SPMM_DECLARE_CFG(launch_cfg_slab32);
SPMM_DECLARE_CFG(launch_cfg_stream64);
SPMM_DECLARE_CFG(launch_cfg_stream32);
SPMM_DECLARE_CFG(launch_cfg_stream16);
#undef SPMM_DECLARE_CFG

bool plan_supported(int token_tile, int variant)
{
    if (token_tile == 128) return variant == 0 || variant == 8 || variant == 16 || variant == 108 || variant == 112;
    if (token_tile == 96) return variant == 0 || variant == 16 || variant == 112;
    if (token_tile == 64) return variant == 101 || variant == 102 || variant == 104 || variant == 112;
    if (token_tile == 32 || token_tile == 16) return variant == 101 || variant == 103 || variant == 104;
    return false;
}

// Pipelined kernel: token tile tm, `waves` row tiles per workgroup.  S token-tile streams per
// row group, enough workgroups to fill every CU once.
static void fill_pipelined(Plan& p, int64_t M, int ntiles, int num_cus, int tm, int waves)
{
    p.token_tile = tm;
    p.waves = waves;
    p.loaders = 0;
    p.row_tiles_per_wave = 1;
    p.simple = 0;
    p.slab = 0;
    p.stream = 0;
    p.n_tok_tiles = (int)((M + tm - 1) / tm);
    p.n_row_groups = (ntiles + waves - 1) / waves;
    int S = num_cus / p.n_row_groups;
    if (S < 1) S = 1;
    if (S > p.n_tok_tiles) S = p.n_tok_tiles;
    if (S >= 8) S -= S % 8;
    p.n_streams = S;
    p.xcd_map = (S % 8 == 0) ? 1 : 0;
    p.workgroups = (int64_t)p.n_row_groups * S;
}

// Simple kernel: tm-token tiles, 8 waves with r row tiles each, one workgroup per (row group, tile).
// Workgroup ids go round the 8 XCDs; which of the two operands an XCD's L2 then holds a slice of:
// map 1 keeps a token tile on one XCD (every XCD reads all of W), map 2 keeps a row group on one
// XCD (every XCD reads all of X): whichever operand is the larger is the one that is sliced.
static void fill_simple(Plan& p, int64_t M, const WeightDims& w, int r, int tm)
{
    const int ntiles = w.ntiles;
    p.token_tile = tm;
    p.waves = 8;
    p.row_tiles_per_wave = r;
    p.simple = 1;
    p.slab = 0;
    p.stream = 0;
    p.n_tok_tiles = (int)((M + tm - 1) / tm);
    p.n_row_groups = (ntiles + p.waves * r - 1) / (p.waves * r);
    p.n_streams = 0;
    const int64_t w_bytes = w.nsteps * (STEP_VAL_BYTES + 4 * STEP_IDX_DWORDS), x_bytes = (int64_t)w.K * M;
    p.xcd_map = (w_bytes > x_bytes) ? 2 : 1;
    p.workgroups = (p.xcd_map == 2) ? (int64_t)8 * ((p.n_row_groups + 7) / 8) * p.n_tok_tiles
                                    : (int64_t)8 * p.n_row_groups * ((p.n_tok_tiles + 7) / 8);
}

// Relative duration of a plan: the longest stream's token tiles times what a tile costs a workgroup
// (its tokens, plus a fixed part per tile, in tokens), plus a start-up term, times the rounds needed
// when there are more workgroups than CUs.  An 8-wave workgroup stages the same activations for half
// as many rows: measured, its token tile takes about two thirds of a 16-wave one (4096x1024, 90 %:
// 33.0 against 25.5 us for twice the tiles).
// With loader waves (4-byte outputs) a tile of 12 compute waves costs about 0.8 of a 16-wave one and one
// of 8 compute waves about 0.6 (3072x768, 4096 tokens, fp32: 22.4 us with 192 workgroups of 16 waves,
// 18.0 us with 256 of 12 + 4; 768x3072: 18.9 us with 8 waves, 16.2 us with 8 + 4 on the same grid).
static double plan_cost(const Plan& p, int num_cus)
{
    const int per_stream = (p.n_tok_tiles + p.n_streams - 1) / p.n_streams;
    const int64_t rounds = (p.workgroups + num_cus - 1) / num_cus;
    double per_token = p.loaders ? (p.waves == 12 ? 0.8 : 0.6) : (p.waves == 16) ? 1.0 : 0.66;
    // 16 waves, 128-token tiles and 6 step slots is the one configuration that does not fit its 128 registers
    // (a few spilled, with scratch traffic to match): 4096x1024 at 80 %, 6144 tokens, runs 33.5 us with it and
    // 30.3 us with four 96-token tiles per stream instead of three of 128
    if (!p.loaders && p.waves == 16 && p.token_tile == 128 && p.max_steps >= 6) per_token = 1.1;
    return (double)rounds * ((double)per_stream * (p.token_tile * per_token + 16.0) + 48.0);
}

Plan make_plan(int64_t M, const WeightDims& w, int num_cus, int force_tm, int variant, bool aligned, int out_bytes)
{
    const int ntiles = w.ntiles, nseg = w.nseg, max_steps_per_segment = w.max_steps_per_segment;
    Plan p{};
    const int max_steps = max_steps_per_segment <= 4 ? 4 : (max_steps_per_segment <= 6 ? max_steps_per_segment : 8);
    p.max_steps = max_steps;
    if (force_tm == 64 && variant == 112) {
        // (weights with more than 6 steps per segment run 8 compute waves, which exist with 128-token tiles)
        fill_pipelined(p, M, ntiles, num_cus, max_steps <= 6 ? 64 : 128, max_steps <= 6 ? 12 : 8);
        p.loaders = 4;
        if (p.max_steps == 5) p.max_steps = 6;
        return p;
    }
    if ((force_tm == 16 || force_tm == 32) && variant == 103) {
        // the short-batch kernel holds K <= 4096 (3072 with 32-token tiles); longer K silently runs
        // the simple kernel
        fill_simple(p, M, w, 1, force_tm);
        p.slab = nseg <= (force_tm == 16 ? SLAB_SEGMENTS : SLAB_SEGMENTS_32);
        return p;
    }
    if ((force_tm == 64 || force_tm == 32 || force_tm == 16) && variant == 104) {
        fill_simple(p, M, w, 1, force_tm);
        p.stream = 1;
        return p;
    }
    if (force_tm == 64 || force_tm == 32 || force_tm == 16) {
        fill_simple(p, M, w, variant - 100, force_tm);
        return p;
    }
    if (variant == 108 || variant == 112) {
        // 12 compute waves have 128 registers each (at most 6 step slots); denser weights take 8
        const int waves = (variant == 112 && max_steps <= 6 ) ? 12 : 8;
        fill_pipelined(p, M, ntiles, num_cus, (waves == 12 && force_tm == 96) ? 96 : 128, waves);
        p.loaders = 4;
        if (p.max_steps == 5) p.max_steps = 6;
        return p;
    }
    // 16 waves have 128 registers each: at most 6 steps per segment; denser weights run with 8
    // waves, 256 registers and half as many rows per workgroup (token tile 128 only).
    if (max_steps > 6 || variant == 8 || (!aligned && force_tm == 0 && variant == 0)) {
        fill_pipelined(p, M, ntiles, num_cus, 128, 8);
    } else if (force_tm == 96 || variant == 16) {
        fill_pipelined(p, M, ntiles, num_cus, force_tm ? force_tm : 128, 16);
        return p;
    } else {
        // Token tile 128 or 96: 96 where it shortens the longest stream (6144 tokens and 4 row
        // groups: 64 tiles of 96 fill the 256 CUs, 48 tiles of 128 leave a quarter idle; measured
        // 10.6 -> 10.2 us and 27.0 -> 26.1 us at 90 %, 14.4 -> 12.4 us and 39.6 -> 33.5 us at 80 %);
        // with 16 row groups four tiles of 96 per stream lose to three of 128 (26.7 against 25.1 us).
        fill_pipelined(p, M, ntiles, num_cus, 128, 16);
        if (force_tm == 0) {
            Plan c{};
            c.max_steps = max_steps;
            fill_pipelined(c, M, ntiles, num_cus, 96, 16);
            if (plan_cost(c, num_cus) < plan_cost(p, num_cus)) p = c;
        }
        // few row groups and few token tiles (BERT-Base shapes, short batches): 8-wave workgroups
        // are twice as many and fill more CUs
        Plan c{};
        c.max_steps = max_steps;
        fill_pipelined(c, M, ntiles, num_cus, 128, 8);
        if (plan_cost(c, num_cus) < plan_cost(p, num_cus)) p = c;
    }
    if (out_bytes == 4 && force_tm == 0 && variant == 0) {
        // 4-byte outputs: the stores of a tile are 4 N M bytes and a wave that stores cannot wait for
        // loads without waiting for them too; workgroups with loader waves keep multiplying meanwhile
        Plan c{};
        c.max_steps = (max_steps == 5) ? 6 : max_steps;
        fill_pipelined(c, M, ntiles, num_cus, 128, 8);
        c.loaders = 4;
        if (p.waves == 8 || plan_cost(c, num_cus) < plan_cost(p, num_cus)) p = c;
        if (max_steps <= 6) {
            // (768x3072, 6144 tokens, 80 %: 28.5 us with 16 waves, 22.5 us with 12 + 4 and 96-token tiles;
            // 768x768, 4096 tokens: 9.3 us with 8 + 4 and 128-token tiles on 192 CUs, 8.3 us with 12 + 4 and 64-token tiles on 256)
            for (int tm = 128; tm >= 64; tm -= 32) {
                fill_pipelined(c, M, ntiles, num_cus, tm, 12);
                c.loaders = 4;
                if (plan_cost(c, num_cus) < plan_cost(p, num_cus)) p = c;
            }
        }
    }
    if (force_tm == 0 && variant == 0 && p.workgroups * 2 <= num_cus) {
        // Small problems (short batches): the persistent kernel cannot fill half the CUs; the
        // simple kernel cuts the work into 128-row x 64-token pieces, one workgroup each, and is
        // the faster one there (768x768, 128..1024 tokens: 5.8-6.0 us against 7.5-7.9 us).
        Plan c{};
        c.max_steps = max_steps;
        fill_simple(c, M, w, 1, 64);
        if ((int64_t)c.n_row_groups * c.n_tok_tiles >= p.workgroups) {   // (its grid is padded to the XCDs)
            p = c;
            // A simple-kernel workgroup is bound by its own CU's LDS (8 waves gathering from one
            // staged segment), so while CUs are idle, narrower token tiles on more CUs finish
            // sooner: the narrowest tile that still gives every workgroup a CU of its own.
            for (int tm = 32; tm >= 16; tm /= 2) {
                fill_simple(c, M, w, 1, tm);
                if ((int64_t)c.n_row_groups * c.n_tok_tiles <= num_cus) p = c;
            }
            // From five K segments on (K > 2048) the short-batch kernel, which fetches its whole
            // slab of activations at once, beats the segment-by-segment loop (768x3072, 32 tokens:
            // 6.4 against 7.3 us); below, its larger fixed cost loses (768x768: 4.9 against 3.8 us).
            if (p.token_tile == 16 && nseg >= 5 && nseg <= SLAB_SEGMENTS) p.slab = 1;
            // (32-token tiles, 768x3072, 1024 tokens: 9.7 against 10.5 us; at 70 %: 13.1 against 13.8 us)
            if (p.token_tile == 32 && nseg >= 5 && nseg <= SLAB_SEGMENTS_32) p.slab = 1;
            // Longest K (seven segments and more) where the slab does not fit or the tile is wider:
            // the streamed kernel (1024x4096, 1024 tokens: 12.8 against 17.4 us at 90 %, 18.6 against
            // 28.2 us at 70 %; 4096x4096, 384 tokens, 70 %: 20.3 against 27.2 us); with fewer segments
            // its longer code costs more than the hidden weight latency saves.
            if (!p.slab && nseg >= 7) p.stream = 1;
        }
    }
    if (!p.simple) {
        // the same choice of the sliced operand as for the simple kernel (fill_simple): all
        // streams of a row group on one XCD when the packed weight is larger than X
        const int64_t w_bytes = w.nsteps * (STEP_VAL_BYTES + 4 * STEP_IDX_DWORDS), x_bytes = (int64_t)w.K * M;
        if (w_bytes > x_bytes && p.n_row_groups % 8 == 0) p.xcd_map = 2;
    }
    return p;
}

int launch_spmm(const Plan& plan, KernelArgs& a, spmm_out_t out_type, int postop, void* stream)
{
    (void)hipGetLastError();   // an error left by an earlier, unrelated call is not this launch's
    a.n_tok_tiles = plan.n_tok_tiles;
    a.n_row_groups = plan.n_row_groups;
    a.n_streams = plan.n_streams;
    a.xcd_map = plan.xcd_map;
    const unsigned block = (unsigned)(plan.waves + plan.loaders) * 64;
    if (plan.simple) {
        const unsigned grid = (unsigned)plan.workgroups;
        const int key = plan.token_tile * 10 + plan.row_tiles_per_wave;
        if (plan.stream) {
            if (a.kc != SEGMENT_ROWS) return (int)hipErrorInvalidValue;
            if (key == 641) launch_cfg_stream64(out_type, postop, grid, 1, block, stream, a);
            else if (key == 321) launch_cfg_stream32(out_type, postop, grid, 1, block, stream, a);
            else if (key == 161) launch_cfg_stream16(out_type, postop, grid, 1, block, stream, a);
            else return (int)hipErrorInvalidValue;
        } else if (plan.slab) {
            if (a.kc != SEGMENT_ROWS) return (int)hipErrorInvalidValue;
            if (key == 161 && a.nseg <= SLAB_SEGMENTS) launch_cfg_slab16(out_type, postop, grid, 1, block, stream, a);
            else if (key == 321 && a.nseg <= SLAB_SEGMENTS_32) launch_cfg_slab32(out_type, postop, grid, 1, block, stream, a);
            else return (int)hipErrorInvalidValue;
        } else if (key == 641) launch_cfg_simple_1(out_type, postop, grid, 1, block, stream, a);
        else if (key == 642) launch_cfg_simple_2(out_type, postop, grid, 1, block, stream, a);
        else if (key == 321) launch_cfg_simple32_1(out_type, postop, grid, 1, block, stream, a);
        else if (key == 161) launch_cfg_simple16_1(out_type, postop, grid, 1, block, stream, a);
        else return (int)hipErrorInvalidValue;
        return (int)hipGetLastError();
    }
    if (a.kc != SEGMENT_ROWS) return (int)hipErrorInvalidValue;
    // 2-D grid: x = token-tile stream, y = row group
    unsigned gx = (unsigned)plan.n_streams, gy = (unsigned)plan.n_row_groups;
    if (plan.xcd_map == 2) { gx = (unsigned)plan.n_row_groups; gy = (unsigned)plan.n_streams; }
    a.tiles_per_stream = plan.n_tok_tiles / plan.n_streams;
    a.tiles_extra = plan.n_tok_tiles % plan.n_streams;
    const int maxs = (plan.waves == 8 && plan.max_steps == 5) ? 6 : plan.max_steps;   // no 8-wave 5-step build
    if (plan.loaders) {
        switch (plan.token_tile * 10000 + plan.waves * 100 + maxs) {
        case 1281204: launch_cfg_fed_128_12_4(out_type, postop, gx, gy, block, stream, a); break;
        case 1281206: launch_cfg_fed_128_12_6(out_type, postop, gx, gy, block, stream, a); break;
        case 1280804: launch_cfg_fed_128_8_4(out_type, postop, gx, gy, block, stream, a); break;
        case 1280806: launch_cfg_fed_128_8_6(out_type, postop, gx, gy, block, stream, a); break;
        case 1280808: launch_cfg_fed_128_8_8(out_type, postop, gx, gy, block, stream, a); break;
        case 961204: launch_cfg_fed_96_12_4(out_type, postop, gx, gy, block, stream, a); break;
        case 961206: launch_cfg_fed_96_12_6(out_type, postop, gx, gy, block, stream, a); break;
        case 641204: launch_cfg_fed_64_12_4(out_type, postop, gx, gy, block, stream, a); break;
        case 641206: launch_cfg_fed_64_12_6(out_type, postop, gx, gy, block, stream, a); break;
        default: return (int)hipErrorInvalidValue;
        }
        return (int)hipGetLastError();
    }
    switch (plan.token_tile * 10000 + plan.waves * 100 + maxs) {
    case 1281604: launch_cfg_128_16_4(out_type, postop, gx, gy, block, stream, a); break;
    case 1281605: launch_cfg_128_16_5(out_type, postop, gx, gy, block, stream, a); break;
    case 1281606: launch_cfg_128_16_6(out_type, postop, gx, gy, block, stream, a); break;
    case 1280804: launch_cfg_128_8_4(out_type, postop, gx, gy, block, stream, a); break;
    case 1280806: launch_cfg_128_8_6(out_type, postop, gx, gy, block, stream, a); break;
    case 1280808: launch_cfg_128_8_8(out_type, postop, gx, gy, block, stream, a); break;
    case 961604: launch_cfg_96_16_4(out_type, postop, gx, gy, block, stream, a); break;
    case 961605: launch_cfg_96_16_5(out_type, postop, gx, gy, block, stream, a); break;
    case 961606: launch_cfg_96_16_6(out_type, postop, gx, gy, block, stream, a); break;
    default: return (int)hipErrorInvalidValue;
    }
    return (int)hipGetLastError();
}

}  // namespace spmm

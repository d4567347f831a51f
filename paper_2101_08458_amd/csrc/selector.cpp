// Tile-shape selector: maps (rows, cols, reduction length) of the implicit GEMM to one
// of the compiled tile shapes plus a grid split of the reduction.  This is the paper's
// tuner (Section III-C.3 and the GPU tuning paragraphs of Section IV-C: accumulator window
// size, fused spatial dimensions, split reduction; "profile and pick") reduced to a rule fitted
// to measurements, since the paper finds that tuning beyond fuse + split adds little
// (Section VI-B).
#include <atomic>

#include "unit_internal.h"

namespace unit {

#define UNIT_TILE_CASE(ID, BM, BN, BKB, WGM, WGN, WGK, MF, NST, OCC) \
    {BM, BN, BKB, WGM, WGN, WGK, MF, NST},
const TileCfg g_tiles[NUM_TILES] = {
#include "tiles.def"
};
const TileCfg g_tiles_fp8[NUM_TILES] = {
#include "tiles_fp8.def"
};
#undef UNIT_TILE_CASE

// Process-wide override of the rule (unit_debug_force_tile): -1 = none.  Set by tests and tuning
// sweeps only; the hot path reads two relaxed atomics.
static std::atomic<int> g_force_tile{-1}, g_force_split{-1};
void force_tile(int tile, int split)
{
    g_force_tile.store(tile, std::memory_order_relaxed);
    g_force_split.store(split, std::memory_order_relaxed);
}

bool tile_is_forced() { return g_force_tile.load(std::memory_order_relaxed) >= 0; }

// Whether tile `t` has a kernel for this B source and operand type: the LDS footprint and the
// vmcnt range of IgemmCfg::FITS, recomputed on the host.
bool tile_fits(int tile, int dtype, int bsrc)
{
    if (tile < 0 || tile >= NUM_TILES) return false;
    const TileCfg &c = (dtype == 4 /* fp8 */ ? g_tiles_fp8 : g_tiles)[tile];
    if (c.bm == 0) return false;                                     // no kernel of this tile for the type
    const int nw = c.wgm * c.wgn * c.wgk, rpi = 1024 / c.bkb;
    const int lpt = c.bm / rpi / nw + c.bn / rpi / nw;
    const long edge = (bsrc == BSRC_NCHWS || bsrc == BSRC_NCHW) ? 1024 : 0;   // (NCHW may become NCHWE)
    const long ring = (long)c.nst * (c.bm + c.bn) * c.bkb + edge;
    const long red = c.wgk > 1 ? (long)c.wgk * c.bm * c.bn * 4 : 0;
    const bool direct = bsrc == BSRC_NCHW || bsrc == BSRC_NCHWS || bsrc == BSRC_NCHWE;
    const int es = (dtype == 1 || dtype == 2) ? 2 : 1;              // fp16 / bf16: two-byte elements
    const int cpr = c.bn * es / 16;                                  // 16-byte chunks per channel row of the B tile
    if (direct && (cpr > 64 || 64 % cpr != 0)) return false;
    return (ring > red ? ring : red) <= 160 * 1024 && (c.nst - 1) * lpt <= 63;
}

static inline int cdiv(long a, long b) { return (int)((a + b - 1) / b); }

TileChoice select_tile(int rows, int cols, int kchunks, int dtype, int bsrc, bool allow_split, int cb)
{
    const int CUS = 256;
    int tile = -1;
    if (rows <= 16) {
        tile = 5;
    } else {
        // largest tile that still gives every compute unit a workgroup
        static const int order[] = {8, 1};
        for (int t : order) {
            const TileCfg &c = g_tiles[t];
            long nt = (long)cdiv(rows, c.bm) * cdiv(cols, c.bn);
            double fill = (double)rows * cols / ((double)nt * c.bm * c.bn);
            // the 256x256 tile's prologue and epilogue only amortise over a long reduction
            if (t == 8 && kchunks < 32) continue;
            if (nt >= CUS * 3 / 4 && fill >= 0.6) { tile = t; break; }
        }
        // Few output rows (<= 64 channels) but very many columns (network stems and first
        // stages at batch >= 8): a 64x64 tile starves its waves (one accumulator each).  The
        // 64x256 tile gives every wave a 64x64 window without wasted rows; for short reductions
        // the 128x128 tile is as fast even with half of its rows empty (they cost no traffic).
        if (tile < 0 && rows <= 64 && (long)cdiv(cols, 256) >= CUS * 3 / 4)
            tile = (kchunks >= 32) ? 6 : 1;
        // small problems are launch- and latency-bound: measured over the ResNet-50 batch-1
        // layers, 64x64 (2x2x2 waves) wins once it yields ~160 workgroups, 32x32 below that (at ~100 the
        // 32x32 tile's ~400 workgroups fill the chip and finish 0.2-0.4 us earlier, unless the reduction is
        // deep, beyond 160 chunks: there the 64x64 tile's fewer bytes per MAC count for more; the 256-channel
        // 3x3 layers of the ResNet-18 chain at batch 8, 100 tiles of 64x64 and 144 chunks, are 1.4 us faster
        // each on 32x32 tiles inside the chain)
        // (a 64x64 tile with 256-byte steps in two stages is 4-18 % faster on deep reductions when a layer
        // is timed alone, but slower inside a sequence of layers, where every launch starts on cold caches)
        if (tile < 0) {
            const long n64 = (long)cdiv(rows, 64) * cdiv(cols, 64);
            tile = (n64 >= 160 || (n64 >= 96 && kchunks > 160)) ? 3 : 4;
        }
    }
    // 64-byte pixels (64 int8 or 32 fp16 channels): the small tile with 64-byte steps.  The shifted direct read
    // needs it (its steps must stay inside one tap); the gather gets one tap per step with it, i.e. the scalar
    // tap walk instead of the per-lane one (config 1, 64 -> 64 channels 3x3 at 56x56: 3.9 -> 3.5 us)
    // (for the gather only while the reduction is at most 2 KiB: beyond that twice the steps cost more than the
    // per-lane tap walk; Table I layers, both types)
    // (also in place of the 64x64 tile on packed activations: the 64-channel 3x3 layers of the ResNet-18 chain at
    // batch 8, 392 tiles of 64x64, are 1 us faster each with one tap per step inside the chain)
    if ((tile == 4 || (tile == 3 && bsrc == BSRC_GATHER)) && cb > 0 && cb % 8 != 0 && cb % 4 == 0 &&
        (bsrc == BSRC_NCHWS || (bsrc == BSRC_GATHER && kchunks <= 128)))
        tile = 9;
    // A 1x1 direct read whose whole reduction is 64 bytes (64 int8 / 32 fp16 channels): one 64-byte step instead of a
    // half-empty 128-byte one (64 -> 256 channels at 56x56, batch 1: -0.5 us per layer against the 64x64 tile)
    if ((tile == 3 || tile == 4) && bsrc == BSRC_NCHW && kchunks <= 4) tile = 9;
    // Few output elements (the 14x14 and 7x7 layers at batch 1): 16x16 tiles with 256-byte steps give most compute
    // units a workgroup of their own without a grid split of the reduction, i.e. without the reduce launch.
    //  * Operand rows that are contiguous reduction bytes (packed activations, plain matmul): from 32 chunks of
    //    reduction on and up to 128 tiles of 32x32, whatever the pixel size -- fastest on 28 of the 32 small Table I
    //    cases (both types; 3.3-5.7 us against 3.9-6.9 us for the best other tile and split), on the stride-2 layers of
    //    the ResNet-50 set and through the ResNet-18 chain; up to 256 tiles of 32x32 when the reduction is 256 chunks
    //    or more (the 512-channel 3x3 layers of that chain at batch 8: 208 tiles, -1.1 us each inside the chain).
    //  * Direct reads: a 16-pixel tile takes 16 bytes from each 128-byte line of a channel row, so its steps cost
    //    0.26-0.38 us against 0.17 us on packed rows; it pays up to 64 tiles of 32x32 and for four to ten steps
    //    (ResNet-50 batch-1 step: -1.1 us on each 256-channel 3x3 layer at 14x14, -0.5 us on 1024 -> 256 at 14x14,
    //    -2.5 us on 2048 -> 512 at 7x7; 512-channel 3x3 at 7x7, 18 steps: as fast split across 32x32 workgroups;
    //    256 -> 1024 at 14x14, 224 tiles: +0.8 us).  The shifted read needs 256-byte pixels (a step stays inside a tap).
    if (tile == 4 || tile == 9) {
        const long n32 = (long)cdiv(rows, 32) * cdiv(cols, 32);
        const bool contiguous = bsrc == BSRC_PLAIN || bsrc == BSRC_GATHER;
        const bool pick = contiguous ? ((n32 <= 128 && kchunks >= 32) || (n32 <= 256 && kchunks >= 256))
                                     : (tile == 4 && n32 <= 64 && kchunks >= 64 && kchunks <= 160 &&
                                        (bsrc != BSRC_NCHWS || (cb > 0 && cb % 16 == 0)));
        if (pick && tile_fits(12, dtype, bsrc)) tile = 12;
    }
    const int forced = g_force_tile.load(std::memory_order_relaxed);
    if (forced >= 0 && forced < NUM_TILES) tile = forced;

    const TileCfg &c = g_tiles[tile];
    const int nch = c.bkb / 16;
    const int ksteps_tile = cdiv(kchunks, nch);    // main-loop steps of the chosen tile
    const int ksteps = cdiv(kchunks, 8);           // the split rules count 128-byte steps whatever the tile's step
    const long nt = (long)cdiv(rows, c.bm) * cdiv(cols, c.bn);
    // Split the reduction across workgroups only for deep reductions with few tiles: each
    // main-loop step of a small tile costs ~0.2 us of DMA latency, while the extra reduce
    // launch costs ~3 us, so it pays from about 24 steps on (slices of ~6 steps).
    int split = 1;
    if (tile == 12) {
        // the 16x16 tile exists to avoid the reduce launch: measured best unsplit up to 20 of its steps (Table I layer 1
        // in fp16, the 512-channel 3x3 layers); only far deeper reductions are cut, into slices of 32 steps
        if (ksteps_tile >= 64) split = ksteps_tile / 32;
    } else if (ksteps >= 24 && nt <= CUS / 2) {
        split = ksteps / 6;
        int cap = (int)(2 * CUS / nt);
        if (split > cap) split = cap;
        if (split < 1) split = 1;
    } else if (bsrc == BSRC_NCHWS && ksteps >= 12 && nt <= CUS / 4) {
        // the shifted direct read has no pack launch in front of it to hide under, and its steps are a
        // little longer (unaligned 16-byte loads): with a quarter of the chip or less busy, slices of
        // about 4 steps measured best (the 14x14 layers)
        split = ksteps / 4;
    }
    const int fs = g_force_split.load(std::memory_order_relaxed);
    if (fs >= 1) split = fs;
    if (!allow_split) split = 1;
    if (split > ksteps_tile) split = ksteps_tile;
    int per = cdiv(ksteps_tile, split);
    split = cdiv(ksteps_tile, per);                // drop empty slices
    TileChoice ch;
    ch.tile = tile;
    ch.split_k = split;
    ch.ksteps_per_split = per;
    ch.workgroups = (int)(nt * split);
    return ch;
}

// Relative cost of one tile of the narrower relatives of the 256 x 256 tile, per unit of reduction, in units of the
// large tile's own cost (measured on matmuls that fill exactly one round of 256 workgroups with each shape).
static const struct { int tile, bn; double cost; } g_tail_tiles[] = {{10, 192, 0.79}, {11, 128, 0.60}};

RangePlan plan_ranges(int rows, int cols, int kchunks, int dtype, int bsrc, bool allow_split, int cb, bool allow_ranges)
{
    RangePlan p;
    p.n = 1;
    p.col_begin[0] = 0;  p.col_end[0] = cols;
    p.col_begin[1] = p.col_end[1] = cols;
    p.choice[0] = select_tile(rows, cols, kchunks, dtype, bsrc, allow_split, cb);
    p.choice[1] = p.choice[0];
    if (!allow_ranges || g_force_tile.load(std::memory_order_relaxed) >= 0) return p;
    if (p.choice[0].tile != 8 || p.choice[0].split_k != 1) return p;
    const int CUS = 256, BN = 256;
    const long tm = cdiv(rows, 256), tn = cdiv(cols, BN), nt = tm * tn;
    if (nt <= CUS || nt % CUS == 0) return p;
    // main range: the column tiles that make whole rounds of workgroups; tail: the rest
    const long n1 = (nt / CUS) * CUS / tm;
    if (n1 <= 0 || n1 >= tn) return p;
    const long c1 = n1 * BN, tail_cols = cols - c1;
    const double plain = (double)cdiv(tm * cdiv(tail_cols, BN), CUS);      // rounds the tail takes as large tiles
    int best = -1;
    double best_cost = 0.92 * plain;                                       // a second launch must pay for itself
    for (unsigned i = 0; i < sizeof g_tail_tiles / sizeof g_tail_tiles[0]; ++i) {
        const long t = tm * cdiv(tail_cols, g_tail_tiles[i].bn);
        if (t <= CUS && g_tail_tiles[i].cost < best_cost && tile_fits(g_tail_tiles[i].tile, dtype, bsrc)) {
            best = (int)i;
            best_cost = g_tail_tiles[i].cost;
        }
    }
    if (best < 0) return p;
    const TileCfg &c = g_tiles[g_tail_tiles[best].tile];
    p.n = 2;
    p.col_end[0] = (int)c1;
    p.choice[0].workgroups = (int)(n1 * tm);
    p.col_begin[1] = (int)c1;  p.col_end[1] = cols;
    p.choice[1].tile = g_tail_tiles[best].tile;
    p.choice[1].split_k = 1;
    p.choice[1].ksteps_per_split = cdiv(kchunks, c.bkb / 16);
    p.choice[1].workgroups = (int)(tm * cdiv(tail_cols, c.bn));
    return p;
}

}  // namespace unit

// Work split of the tiled GEMM kernels: which output tiles a persistent workgroup computes, in which order.
// Shared by the kernels (device) and the launch code (host); the host can replay the whole schedule
// (batq_debug_tile_schedule) so that it can be checked without a GPU.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace batq {

constexpr int kTile = 256;                 // tile rows
constexpr int kStrip = 64;                 // tile columns come in strips of 64

struct TilePlan {
    int tiles_m;      // row panels of 256
    int strips_n;     // column strips of 64
    int bands;        // column bands (1, 2, 4 or 8)
    int workers;      // workgroups launched, a multiple of 8
    int ksplit;       // parts the K groups are cut into (1: every tile runs over all of K)
    int groups;       // K groups of 256 elements
    int pair;         // 64-column strips per scheduling unit: 1, or 2 when tiles must be an even number of strips
                      // wide (gated output; strips_n then counts units of 128 columns)
};

struct Tile {
    int m0, n0, nj;
    int part, g0, ng;   // K part, its first K group and its number of K groups
};

// A workgroup's walk through its share [cur, end) of the linear order: K part by K part, inside a part the strip
// order (column bands -> row panels -> strips).  The position is decoded once (divisions) and then advanced tile by
// tile with additions and compares only: the kernels take the next tile between an epilogue and the next main loop,
// where every instruction is on the critical path (the same walk decoded from scratch for every tile cost ~900 cycles
// per tile).
struct TileWalk {
    int cur, end;            // position and end of the share, in scheduling units over all K parts
    int part, at;            // K part of `cur` and position inside it
    int b, bs, width;        // column band of `cur`: index, first unit, units
    int p, sl;               // row panel and unit inside the band's panel row
    int g0, ng;              // K groups of `part`
    int lead;                // narrower tiles still to be put in front of the wider ones (see walk_begin)
};

__host__ __device__ inline void walk_set_band(const TilePlan& pl, TileWalk& w) {
    w.bs = w.b * pl.strips_n / pl.bands;
    w.width = (w.b + 1) * pl.strips_n / pl.bands - w.bs;
}
__host__ __device__ inline void walk_set_part(const TilePlan& pl, TileWalk& w) {
    w.g0 = pl.groups * w.part / pl.ksplit;
    w.ng = pl.groups * (w.part + 1) / pl.ksplit - w.g0;
}
// Tiles a run of `run` units is cut into: at most 4 strips = 4 / pair units each.
__host__ __device__ inline int run_tiles(const TilePlan& pl, int run) {
    const int shift = pl.pair == 2 ? 1 : 2;
    return (run + (1 << shift) - 1) >> shift;
}
// Start of the walk over [cur, end) by workgroup `block`.
// A run of units is cut into tiles of near-equal width, i.e. of two widths one unit apart.  Workgroups whose shares
// are alike would all reach their epilogues at the same moments, and the whole chip would then write its output
// in bursts (the write path, not the compute units, sets the length of such an epilogue) and not at all in
// between.  So the workgroups of an XCD take turns in how many of the narrower tiles of their first run they put in
// front of the wider ones: with 3 narrow tiles of 10 the four classes run a quarter of a tile apart.  Workgroups that
// stream the same weight columns (same place in their row panel, 8 apart inside the XCD) are in the same class.
__host__ __device__ inline void walk_begin(const TilePlan& pl, int block, int cur, int end, TileWalk& w) {
    w.cur = cur;
    w.end = end;
    const int per_part = pl.tiles_m * pl.strips_n;
    w.part = pl.ksplit > 1 ? cur / per_part : 0;
    w.at = cur - w.part * per_part;
    w.b = 0;
    while (w.b + 1 < pl.bands && w.at >= pl.tiles_m * ((w.b + 1) * pl.strips_n / pl.bands)) ++w.b;
    walk_set_band(pl, w);
    const int local = w.at - pl.tiles_m * w.bs;
    w.p = local / w.width;
    w.sl = local - w.p * w.width;
    walk_set_part(pl, w);
    int run = end - cur;
    if (per_part - w.at < run) run = per_part - w.at;
    if (w.width - w.sl < run) run = w.width - w.sl;
    w.lead = 0;
    if (run > 0) {
        const int nt = run_tiles(pl, run);
        const int wide = nt == 1 ? run : (run + nt - 1) / nt;
        const int narrow = nt * wide - run;                 // tiles of width wide - 1 in the run
        w.lead = (block >> 3) & 3;
        while (w.lead > narrow) w.lead -= narrow + 1;
    }
}
// Takes the next tile off the walk: at most 4 strips of what is left of the share in this row panel of the band (a
// tile does not reach into the next panel, band or K part), the run cut into tiles of near-equal width.
__host__ __device__ inline bool next_tile(const TilePlan& pl, TileWalk& w, Tile& t) {
    if (w.cur >= w.end) return false;
    const int per_part = pl.tiles_m * pl.strips_n;
    int run = w.end - w.cur;
    if (per_part - w.at < run) run = per_part - w.at;
    if (w.width - w.sl < run) run = w.width - w.sl;       // units left in this row panel of the band
    const int nt = run_tiles(pl, run);                    // tiles the run is cut into, near-equal widths
    int units = nt == 1 ? run : (run + nt - 1) / nt;
    if (w.lead > 0 && units * nt != run) {                // a narrower tile first
        --units;
        --w.lead;
    }
    t.nj = units * pl.pair;
    t.m0 = w.p * kTile;
    t.n0 = (w.bs + w.sl) * kStrip * pl.pair;
    t.part = w.part;
    t.g0 = w.g0;
    t.ng = w.ng;
    // advance
    w.cur += units;
    w.at += units;
    w.sl += units;
    if (w.sl == w.width) {
        w.sl = 0;
        if (++w.p == pl.tiles_m) {
            w.p = 0;
            if (++w.b == pl.bands) {                      // the part is done (at == per_part)
                w.b = 0;
                w.at = 0;
                ++w.part;
                if (w.cur < w.end) walk_set_part(pl, w);
            }
            if (w.cur < w.end) walk_set_band(pl, w);
        }
    }
    return true;
}

// Column bands: with b bands an XCD's block spans 1/b of N and b/8 of M.  A workgroup walks its strips along N
// inside a row panel, tile round by tile round (a tile is at most 4 strips wide); the workgroups of an XCD do so in
// step, so a round streams the block's A rows once more (they do not survive a round in the 4 MiB L2: measured on
// 8192 x 3584 x 18944 with 4 bands, 10 rounds: 746 MB fetched where one pass over the blocks would be 140 MB)
// and its share of the B columns once.  The bytes all L2s pull are therefore proportional to
// rounds * b * M + (8 / b) * N; take the b that minimises it.
inline int choose_bands(int M, int N, int strips_n, int tiles_m, int workers) {
    const long strips = (long)tiles_m * strips_n;
    const long per_worker = (strips + workers - 1) / workers;
    const long rounds = per_worker > 4 ? (per_worker + 3) / 4 : 1;
    int best = 1;
    double best_cost = 1e300;
    for (int b = 1; b <= 8; b *= 2) {
        if (b > strips_n) break;
        const double cost = (double)rounds * b * M + (8.0 / b) * N;
        if (cost < best_cost) {
            best_cost = cost;
            best = b;
        }
    }
    return best;
}


// The share of the linear order that workgroup `block` of `pl.workers` works on: workgroups go to the 8 XCDs
// round-robin, so workgroup b takes share (b % 8) * (workers / 8) + b / 8 and the shares of one XCD are
// contiguous.
__host__ __device__ inline void worker_share(const TilePlan& pl, int block, int& cur, int& end) {
    const int per_xcd = pl.workers >> 3;
    const int share = (block & 7) * per_xcd + (block >> 3);
    const int64_t total = (int64_t)pl.tiles_m * pl.strips_n * pl.ksplit;
    if (total < (1 << 20)) {                    // the usual case: 32-bit products and divisions (workers <= 2^11)
        const uint32_t t32 = (uint32_t)total, wk = (uint32_t)pl.workers;
        cur = (int)(t32 * (uint32_t)share / wk);
        end = (int)(t32 * (uint32_t)(share + 1) / wk);
        return;
    }
    cur = (int)(total * share / pl.workers);
    end = (int)(total * (share + 1) / pl.workers);
}

// K parts wanted for a plan without them: fewer strips than half the workgroups (few rows, narrow N) and a
// long K.  A part keeps at least 12 K groups: below that the partial sums' round trip costs more than the
// idle compute units.  `part_bytes` = partial-sum bytes of one part, `scratch_bytes` = what is available.
inline int choose_ksplit(const TilePlan& pl, size_t part_bytes, size_t scratch_bytes) {
    const int strips = pl.tiles_m * pl.strips_n;
    int ksplit = pl.workers / strips;
    if (pl.groups / 12 < ksplit) ksplit = pl.groups / 12;
    if (ksplit > 8) ksplit = 8;
    while (ksplit > 1 && (size_t)ksplit * part_bytes > scratch_bytes) --ksplit;
    return ksplit < 1 ? 1 : ksplit;
}

// Plan of a launch without K parts (ksplit = 1); `glu`: gated output, tiles an even number of strips wide.
inline TilePlan make_plan(int M, int N, int nb, int cus, bool glu) {
    TilePlan pl;
    pl.pair = glu ? 2 : 1;
    pl.tiles_m = (M + kTile - 1) / kTile;
    pl.strips_n = (N + kStrip * pl.pair - 1) / (kStrip * pl.pair);
    pl.workers = 8 * (cus / 8 > 1 ? cus / 8 : 1);       // one persistent workgroup per compute unit
    pl.bands = choose_bands(M, N, pl.strips_n, pl.tiles_m, pl.workers);
    pl.ksplit = 1;
    pl.groups = (nb + 7) / 8;
    return pl;
}

}  // namespace batq

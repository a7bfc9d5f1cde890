#include <math.h>
#include <stdio.h>
#include <string.h>

#include "select.h"

namespace mg {
namespace {

int32_t find(const std::vector<KernelEntry> &table, const char *name)
{
    for (size_t i = 0; i < table.size(); ++i)
        if (strcmp(table[i].name, name) == 0) return static_cast<int32_t>(i);
    return -1;
}

bool try_pick(const std::vector<KernelEntry> &table, const Problem &p, int64_t alignment, const char *name,
              int split, int32_t *kernel, int32_t *out_split)
{
    const int32_t id = find(table, name);
    if (id < 0 || !table[id].legal || !table[id].legal(p, split, alignment)) return false;
    *kernel = id;
    *out_split = split;
    return true;
}

// MFMA kernel of tile `tag` for this problem's operand contiguity: the fast flavour if the problem
// is aligned and made of whole tiles, else the edge flavour.
bool try_mfma(const std::vector<KernelEntry> &table, const Problem &p, int64_t alignment, const char *tag, int split,
              int32_t *kernel, int32_t *out_split)
{
    char name[96];
    const char *contig = p.a_trans ? (p.b_trans ? "kn" : "kk") : (p.b_trans ? "mn" : "mk");
    // operands padded to whole tiles and the caller's own C (Problem::clip_m, clip_n): the 256 x 256 and the 128 x 128
    // direct-to-LDS kernels have a flavour whose epilogue checks bounds, nothing else has
    if (p.clip_m != 0 || p.clip_n != 0) {
        if (strcmp(tag, "hdma16_256x256x64_w2x4") == 0)
            snprintf(name, sizeof name, "%s_256x256x64_w2x4_%s", p.b_trans ? "hdma16c" : "hpp16c", contig);
        else if (strcmp(tag, "hdma16_128x128x64_w2x4") == 0)
            snprintf(name, sizeof name, "hdma16c_128x128x64_w2x4_%s", contig);
        else
            return false;
        return try_pick(table, p, alignment, name, split, kernel, out_split);
    }
    // with B contiguous along k the 256 x 256 direct-to-LDS tile has a faster schedule (wavefronts taking turns:
    // 4096^3 102 -> 99 us, 8192^3 820 -> 747 us, 2048^3 42 -> 38 us)
    if (!p.b_trans && strcmp(tag, "hdma16_256x256x64_w2x4") == 0) {
        snprintf(name, sizeof name, "hpp16_256x256x64_w2x4_%s", contig);
        if (try_pick(table, p, alignment, name, split, kernel, out_split)) return true;
    }
    snprintf(name, sizeof name, "%s_%s", tag, contig);
    if (try_pick(table, p, alignment, name, split, kernel, out_split)) return true;
    // the register-staged 256 x 256 tile has its bounds-checked flavour on eight wavefronts only (on four, 256
    // accumulators per lane leave the checked loads no registers).  Ragged FP16 cubes in place, us, this flavour /
    // the best smaller tile: 3000 66-94 / 91-94, 5002 255-308 / 342-357, 4104 198-248 / 200-202, 2050 52-67 / 38-43
    // (the estimate below ranks all four the right way round)
    if (strcmp(tag, "hmfma_256x256x64_w2x2") == 0) tag = "hmfma_256x256x64_w2x4";
    snprintf(name, sizeof name, "%s_%s_edge", tag, contig);
    return try_pick(table, p, alignment, name, split, kernel, out_split);
}

struct TileChoice {
    const char *tag;
    int bm, bn, bk;
    float ceiling;       // Mflop/us per compute unit with enough resident work-groups
    float per_group;     // ... contributed by each resident work-group
    int resident;        // work-groups a compute unit holds at once
};

constexpr int kComputeUnits = 256;

// Split-K factor for a grid of `blocks` work-groups that each walk `ktiles` K-tiles.  From the sweep:
// a handful of blocks should be split until every compute unit has two (when K has >= 16 tiles and each
// slice keeps >= 4 of them); a grid that fills the chip less than four times over gains from splitting only when K
// is long (each slice keeps >= 24 K-tiles), because the reduce pass costs a launch and a round trip of
// the partial sums; otherwise no split.
int pick_split(int64_t blocks, int64_t ktiles)
{
    int64_t split = 1;
    if (blocks <= 64 && ktiles >= 16) {
        split = ceil_div(2 * kComputeUnits, blocks);
        if (split > ktiles / 4) split = ktiles / 4;
    } else if (blocks < 4 * kComputeUnits && ktiles >= 48) {
        split = ceil_div(4 * kComputeUnits, blocks);
        if (split > ktiles / 24) split = ktiles / 24;
    }
    if (split > 16) split = 16;
    return split < 1 ? 1 : static_cast<int>(split);
}

// Slices of the sum for a matrix-vector product.  Measured: the axpy kernel (32 KB of loads in flight per
// work-group) is fastest with about two work-groups per compute unit, the dot kernel (16 KB) with four; more
// gain nothing and the reduce pass costs.  Each slice keeps at least four rounds of loads, and the partial
// sums must fit the workspace.
int pick_gemv_split(const mg_config &cfg, int64_t outputs, int64_t k, size_t workspace_bytes)
{
    const bool dot = cfg.lds_bytes == 0;
    const int64_t wanted = (dot ? 4 : 2) * kComputeUnits;
    const int64_t groups = ceil_div(outputs, cfg.tile_m);
    if (2 * groups > wanted) return 1;
    int64_t split = ceil_div(wanted, groups);
    if (split > k / (4 * cfg.tile_k)) split = k / (4 * cfg.tile_k);
    if (split > 256) split = 256;
    const int64_t fits = static_cast<int64_t>(workspace_bytes / (static_cast<size_t>(outputs) * sizeof(float)));
    if (split > fits) split = fits;
    return split < 1 ? 1 : static_cast<int>(split);
}

}  // namespace

void select_config(const std::vector<KernelEntry> &table, const Problem &p, int64_t alignment, size_t workspace_bytes,
                   int32_t *kernel, int32_t *split)
{
    *kernel = -1;
    *split = 1;
    const bool f32 = p.dtype == MG_F32;
    if (p.alpha == 0.f || p.k == 0) {
        try_pick(table, p, alignment, f32 ? "scale_f32" : "scale_f16", 1, kernel, split);
        return;
    }
    if (p.m == 1 || p.n == 1) {
        // short rows, thousands of them: four rows per wavefront keep enough loads in flight (long rows a power
        // of two apart are slower that way than one by one)
        const bool many = p.m * p.n >= 16 * kComputeUnits && p.k * static_cast<int64_t>(p.elem()) <= 4096;
        const char *names[2] = {f32 ? (many ? "gemv_dot4_f32" : "gemv_dot_f32") : (many ? "gemv_dot4_f16" : "gemv_dot_f16"),
                                f32 ? "gemv_axpy_f32" : "gemv_axpy_f16"};
        for (const char *name : names) {
            if (!try_pick(table, p, alignment, name, 1, kernel, split)) continue;
            const int want = pick_gemv_split(table[*kernel].cfg, p.m * p.n, p.k, workspace_bytes);
            if (want > 1) try_pick(table, p, alignment, name, want, kernel, split);
            return;
        }
    }
    // Problems of at most one 32 x 32 block per compute unit and a short sum: the kernel whose eight wavefronts share
    // the sum of one block (tiny.hip) beats the macro tiles' software pipeline, which never fills, and saves the
    // second launch of a sliced sum.  Measured, shared-sum kernel against the best macro tile (with slices), us:
    // FP32 256^3 4.8 / 6.8, 512^3 7.0 / 9.7, (256 | 384 | 512)^2 x 768: 8.9 / 9.2 | 10.0 | 10.8, x 1024: 11.3 / 10.0 |
    // 13.8 | 11.8, x 1536: 15.3 / 11.4 | 15.3 | 14.2; FP16 with B along k, (256^2 | 384^2 | 512^2 | 512 x 196 |
    // 256 x 784) x 1024: 5.8 / 6.7 | 5.8 / 6.6 | 6.1 / 6.7 | 5.8 | 5.9, x 2048: 8.7 / 9.0 | 8.8 / 8.9 | 9.6 / 9.7 |
    // 8.7 / 10.7 | 8.8 / 12.9, x 3072: 11.6 / 10.3 | 11.6 / 13.1 | 12.4 / 11.2 | 11.6 / 11.5 | 13.7 / 14.2.
    // (with fringe rows / columns taken off, the tiles cover tm x tn of C)
    const int64_t tm = p.m - p.fringe_m, tn = p.n - p.fringe_n;
    const int64_t blocks32 = ceil_div(p.m, 32) * ceil_div(p.n, 32);
    const char *order_tag = p.a_trans ? (p.b_trans ? "kn" : "kk") : (p.b_trans ? "mn" : "mk");
    const bool few_blocks = p.shape == MG_SHAPE_GENERAL && blocks32 <= kComputeUnits && p.m > 1 && p.n > 1;
    if (f32 && few_blocks && p.k >= 64 && p.k <= (blocks32 > 64 ? 1024 : 768)) {
        char name[48];
        snprintf(name, sizeof name, "stiny_32x32_%s", order_tag);
        if (try_pick(table, p, alignment, name, 1, kernel, split)) return;
    }
    if (!f32 && few_blocks && !p.b_trans && p.k >= 768 && p.k <= 2560) {
        char name[48];
        snprintf(name, sizeof name, "htiny_32x32_%s", order_tag);
        if (try_pick(table, p, alignment, name, 1, kernel, split)) return;
    }
    if (p.m >= 16 && p.n >= 16) {
        // The macro tile (and number of K slices) with the smallest estimated time, see `estimate` below: a chip
        // that is not full runs ceil(tiles / 256) work-groups per compute unit at a rate that grows with them up to
        // the kernel's ceiling; a full chip works through rounds of 256 x resident work-groups.  Rates (Mflop/us per
        // compute unit: ceiling, per resident work-group) and the number of resident work-groups are fitted to a
        // scan of every tile over problems of 256 to 4608 tiles in the four operand orders, less 2.5 us per launch
        // (what a run of any length costs on top; common to all candidates, so not part of the estimate); partial
        // tiles of ragged problems count as whole ones.  The direct-to-LDS kernels need whole tiles and 16-byte aligned
        // operands; where they are illegal the next best estimate is tried.
        static const TileChoice f16_tiles[] = {{"hdma16_256x256x64_w2x4", 256, 256, 64, 4.88f, 4.83f, 1},
                                               {"hdma16_256x128x64_w4x2", 256, 128, 64, 3.93f, 3.65f, 1},
                                               {"hdma16_128x128x64_w2x4", 128, 128, 64, 4.07f, 2.75f, 2},
                                               {"hmfma_256x256x64_w2x2", 256, 256, 64, 4.54f, 4.40f, 1},
                                               {"hmfma_256x128x64_w2x2", 256, 128, 64, 3.72f, 3.72f, 1},
                                               {"hmfma_128x128x64_w2x2", 128, 128, 64, 3.61f, 3.0f, 2},
                                               {"hmfma_128x64x64_w2x2", 128, 64, 64, 2.85f, 1.87f, 3},
                                               {"hmfma_64x64x64_w2x2", 64, 64, 64, 2.30f, 1.65f, 5}};
        // The register-staged FP16 kernels transpose operands that are not contiguous along k on their way to
        // LDS; the smaller the tile, the more that shows.  Measured rates relative to the (m, k) order (A along m,
        // B along k; tiles up to 128 x 64 / up to 256 x 128 / 256 x 256): both operands along k 1.10 / 1.06 / 1.02,
        // A along m and B along n 0.93 / 0.97 / 0.98.
        auto staged_f16 = [&](const TileChoice &t) {
            const int cls = t.bm * t.bn <= 128 * 64 ? 0 : (t.bm * t.bn <= 256 * 128 ? 1 : 2);
            static const double both_k[3] = {1.10, 1.06, 1.02}, neither_k[3] = {0.93, 0.97, 0.98};
            if (p.a_trans && !p.b_trans) return both_k[cls];
            if (!p.a_trans && p.b_trans) return neither_k[cls];
            return 1.0;
        };
        // FP32: a single work-group keeps the MFMA pipes of its compute unit nearly busy, so work-groups that share
        // a compute unit take turns rather than overlap (128 x 128 at k = 2048: 256 / 288 / 512 / 768 / 1024 tiles
        // take 128 / 233 / 249 / 368 / 474 us): rounds of 256 tiles whatever the tile, at a rate that rises from
        // `per_group` (one round) towards `ceiling` (many), plus what a round of small tiles costs on top
        // (0 / 0 / 1 / 2 / 1.8 us from the largest tile to the smallest: first loads and the epilogue).
        // The two tiles of which a compute unit holds a single work-group run with eight wavefronts (two per SIMD:
        // one hides the other's barrier and LDS waits; 4096^3 in the steady power state 1036 -> 932 us for 256 x 256,
        // 973 -> 950 us for 256 x 128; the four-wavefront variants stay in the table).
        // Rates: turns * tile flops / time of every tile on the squares 1024^3 to 6144^3 (the four operand orders run
        // alike since the operands along m / n keep their memory layout in LDS): one turn gives `per_group`, many
        // turns `ceiling`.
        static const TileChoice f32_tiles[] = {{"smfma_256x256x32_w2x4", 256, 256, 32, 0.591f, 0.591f, 1},
                                               {"smfma_256x128x32_w4x2", 256, 128, 32, 0.587f, 0.583f, 1},
                                               {"smfma_128x128x32_w2x2", 128, 128, 32, 0.588f, 0.566f, 2},
                                               {"smfma_128x64x32_w2x2", 128, 64, 32, 0.582f, 0.54f, 3},
                                               {"smfma_64x64x32_w2x2", 64, 64, 32, 0.571f, 0.565f, 5}};
        static const double f32_round_cost[5] = {0.0, 0.0, 1.0e6, 2.0e6, 1.8e6};
        const TileChoice *tiles = f32 ? f32_tiles : f16_tiles;
        const int count = f32 ? 5 : 8;
        bool tried[8] = {false, false, false, false, false, false, false, false};
        // estimated time (in 1e-6 us) of tile i with the sum cut into `slices`
        auto estimate = [&](int i, int slices) {
            const int64_t blocks = ceil_div(tm, tiles[i].bm) * ceil_div(tn, tiles[i].bn) * slices;
            const double tile_flops = 2.0 * tiles[i].bm * tiles[i].bn * static_cast<double>(p.k) / slices;
            const int64_t full = static_cast<int64_t>(kComputeUnits) * tiles[i].resident;   // work-groups the chip holds
            double order = 1.0;
            if (!f32 && tiles[i].tag[1] == 'm') order = staged_f16(tiles[i]);
            // sliced sums run the large register-staged tiles about a tenth below their rate (256 x 8192 x 8192 with
            // both operands along k in four slices: 53-55 us against 48 us on the direct-to-LDS tile of that size)
            if (!f32 && tiles[i].tag[1] == 'm' && slices > 1 && tiles[i].bm * tiles[i].bn >= 256 * 128) order *= 0.9;
            // the 128 x 128 direct-to-LDS tile is slower with A along k (3.7-3.8 against 4.0)
            if (!f32 && i == 2 && p.a_trans) order = 0.94;
            // ragged or unaligned FP16 problems run the bounds-checked flavour, which costs the smaller tiles more
            // (rates against the whole-tile flavour: 0.75 for 256 x 256 and 256 x 128, about 0.5 for 128 x 128
            // and below; FP32: see below)
            const bool ragged = tm % tiles[i].bm || tn % tiles[i].bn || p.k % tiles[i].bk || tm != p.m || tn != p.n;
            // (operands whose rows start on dwords run their whole K-tiles on the fast schedule: fitted to ragged cubes of
            // 1300 to 5002, (4100, 4100, 512) and (8200, 1030, 2050), every bounds-checked tile forced: the eight-wavefront
            // 256 x 256 tile at its whole-tile rate, 256 x 128 at 0.77, 128 x 128 at 0.75 alone on a compute unit and 0.9
            // with a second work-group to hide the checked part behind)
            const bool dword_rows = !f32 && p.lda % 2 == 0 && p.ldb % 2 == 0;
            if (!f32 && ragged) {
                const int area = tiles[i].bm * tiles[i].bn;
                if (!dword_rows) order *= area < 256 * 128 ? 0.6 : 0.7;
                else if (area >= 256 * 256) order *= 1.0;
                else if (area >= 256 * 128) order *= 0.77;
                else if (area >= 128 * 128) order *= blocks > kComputeUnits ? 0.9 : 0.75;
                else order *= 0.6;
            }
            // rate of a compute unit that holds u work-groups at once: ceiling * (1 - (1 - per_group / ceiling)^u)
            // (measured on the 64 x 64 FP16 tile: 1.33 / 1.85 / 2.02 / 2.11 for u = 1..4, the formula gives
            // 1.31 / 1.86 / 2.09 / 2.18)
            auto shared_rate = [&](int64_t u) {
                const double idle = 1.0 - (tiles[i].per_group < tiles[i].ceiling ? tiles[i].per_group / tiles[i].ceiling : 1.0);
                return tiles[i].ceiling * (1.0 - pow(idle, static_cast<double>(u)));
            };
            double time;
            if (f32) {
                // work-groups take turns on a compute unit: ceil(blocks / 256) turns of one tile each, whether the
                // compute units hold them all at once or are refilled as work-groups retire (squares of 1024 to 6144
                // on every tile: within 6 % of this, the small tiles a little better where the last turn is thin)
                const double rounds = static_cast<double>(ceil_div(blocks, kComputeUnits));
                const double up = ceil(rounds);
                // (the bounds-checked flavour runs its whole K-tiles on the fast flavour's schedule and the end of the sum on
                // checked loads: 0.75 of these rates for a single turn, which has no other work-group's arithmetic to hide
                // the checked part behind, 0.85 for two or more work-groups per compute unit; and every further work-group
                // of a compute unit adds half a turn's fixed cost.  From 64 x 64 tiles, us measured / this estimate:
                // (1000, 1001, 999) unsplit 21.5 / 21.1, two slices 27.0 / 26.7; (4097, 129, 4095) less its fringe unsplit
                // 71 / 81, two slices 46.7 / 47.5, four 46.2 / 44.7, eight 54.9 / 48.4; (1025, 1030, 1000) less its fringe
                // row unsplit 36.3 / 36.6, two slices 35.2 / 37.1, four 38.1 / 36.8)
                const double rate = (tiles[i].ceiling - (tiles[i].ceiling - tiles[i].per_group) / up) * (ragged ? (up <= 1.0 ? 0.75 : 0.85) : 1.0);
                // (work-groups that are resident together pay the fixed cost of a turn once)
                time = rounds * tile_flops / rate + (blocks <= full ? (ragged ? 1.0 + 0.5 * (rounds - 1.0) : 1.0) : rounds) * f32_round_cost[i];
            } else if (blocks < full) {
                // the chip is not full: ceil(blocks / 256) work-groups share a compute unit
                const int64_t per_unit = ceil_div(blocks, kComputeUnits);
                double rate = shared_rate(per_unit);
                // FP16 runs against the power limit: when some compute units hold fewer work-groups than the
                // busiest ones (or none), the busy ones clock higher.  With `load` = the chip's summed rate as a
                // fraction of the rate with every compute unit as busy as the busiest, the gain is load^-e, at
                // most 1.4; e fitted per kernel: 256 x 256 direct-to-LDS 0.55 (144 tiles at 3072^3 run at 6.7
                // Mflop/us per compute unit against 4.8 on a full chip), 256 x 128 0.3 (direct-to-LDS and
                // register-staged), 128 x 128 direct-to-LDS 1.3 when the busiest compute units hold two work-groups
                // (324 tiles at 2304^3: 4.8 Mflop/us against 3.6) but 0.1 with one, the smaller register-staged
                // kernels 0.1; the bounds-checked flavour shows no gain; the 128 x 128 direct-to-LDS tile at most 1.2
                if (!ragged || (dword_rows && i == 3)) {
                    const int64_t busiest = blocks - static_cast<int64_t>(kComputeUnits) * (per_unit - 1);
                    const double lower = per_unit > 1 ? shared_rate(per_unit - 1) : 0.0;
                    const double load = (static_cast<double>(busiest) * rate + static_cast<double>(kComputeUnits - busiest) * lower) /
                                        (static_cast<double>(kComputeUnits) * rate);
                    const double exponent = i == 0 ? 0.55 : (i == 2 ? (per_unit > 1 ? 1.3 : 0.1) : (tiles[i].bm == 256 ? 0.3 : 0.1));
                    const double boost = pow(load, -exponent);
                    const double most = i == 2 ? 1.2 : 1.4;
                    rate *= boost < most ? boost : most;
                }
                time = static_cast<double>(per_unit) * tile_flops / (rate * order);
            } else {
                // whole rounds of `full` work-groups at the ceiling, then the rest.  One work-group per compute
                // unit quantises sharply (576 tiles take three rounds).  FP16 kernels with several resident
                // work-groups: the rest is a round of its own with u = ceil(rest / 256) work-groups per compute
                // unit at their shared rate, four fifths of it exposed (it starts while the round before drains);
                // measured at k = 2048, 512 / 768 / 1024 / 1280 tiles: 128 x 128 direct-to-LDS 37 / 59 / 70 / 91 us
                // (this model: 34 / 57 / 68 / 91), register-staged 41 / 61 / 83 / 104 (38 / 58 / 76 / 96).  The
                // fastest FP16 kernel is an exception of its own: its partial last round runs on fewer compute
                // units at a higher clock (400 tiles take 1.7 rounds' time, 576 tiles 2.5)
                const double x = static_cast<double>(blocks) / static_cast<double>(full);
                const double whole = floor(x);
                const double round_time = tiles[i].resident * tile_flops / (tiles[i].ceiling * order);
                if (x == whole) time = x * round_time;
                else if (i == 0) time = (x + 0.25) * round_time;
                else if (tiles[i].resident == 1) time = (whole + 1.0) * round_time;
                else {
                    const int64_t rest = blocks - static_cast<int64_t>(whole) * full;
                    const int64_t u = ceil_div(rest, kComputeUnits);
                    time = whole * round_time + 0.8 * static_cast<double>(u) * tile_flops / (shared_rate(u) * order);
                }
            }
            // split-K: the partial sums are written and read back (8 bytes per slice and output at ~4 TB/s) by
            // a second launch (2.5 us; 4 us behind the bounds-checked FP32 flavour, fitted with the rates above)
            if (slices > 1) time += 1.0e6 * ((f32 && ragged ? 4.0 : 2.5) + (4.0 * slices + 8.0) * static_cast<double>(p.m) * static_cast<double>(p.n) / 4.0e6);
            return time;
        };
        for (int attempt = 0; attempt < count; ++attempt) {
            int best = -1, best_slices = 1;
            double best_time = 0.0;
            double free_time = 0.0;          // best estimate with all the workspace one could wish for, and its slices
            int free_slices = 0;
            for (int i = 0; i < count; ++i) {
                if (tried[i]) continue;
                // FP32 with a very short K is bound by the traffic of C, which the large tiles overlap worst (one
                // epilogue per compute unit at a time): (8192, 8192, 64) with beta = 1 takes 223 us on 256 x 256
                // tiles, 155-175 us on 64 x 64
                if (f32 && p.k <= 128 && tiles[i].bm * tiles[i].bn > 128 * 64) continue;
                const bool last = i == count - 1;
                const int64_t ktiles = ceil_div(p.k, tiles[i].bk);
                const int64_t blocks = ceil_div(tm, tiles[i].bm) * ceil_div(tn, tiles[i].bn);
                // slices tried: none; for the smallest tile the factor of the sweep's rule; for grids that do not
                // fill the chip powers of two that leave every slice at least four K-tiles (never with a shape hint)
                int options[6] = {1, 0, 0, 0, 0, 0};
                int n_options = 1;
                if (p.shape == MG_SHAPE_GENERAL) {
                    if (last) options[n_options++] = pick_split(blocks, ktiles);
                    if (blocks < 2 * kComputeUnits)
                        for (int sl = 2; sl <= 16 && ktiles / sl >= 4; sl *= 2) options[n_options++] = sl;
                }
                for (int o = 0; o < n_options; ++o) {
                    const int sl = options[o];
                    if (sl < 1 || (o > 0 && sl == 1)) continue;
                    const double time = estimate(i, sl);
                    if (free_slices == 0 || time < free_time) { free_slices = sl; free_time = time; }
                    if (sl > 1 && static_cast<size_t>(sl) * p.m * p.n * sizeof(float) > workspace_bytes) continue;
                    if (best < 0 || time < best_time) { best = i; best_slices = sl; best_time = time; }
                }
            }
            if (best < 0) break;
            // FP16, other orders and shorter sums: where the macro tiles would cut a sum of at most three 512-wide chunks
            // into slices (a second launch that adds the partial sums), the shared-sum kernel does it in one
            // (whether or not the caller brought the workspace for the slices)
            if (!f32 && attempt == 0 && free_slices > 1 && p.shape == MG_SHAPE_GENERAL && blocks32 <= kComputeUnits && p.k <= 1536) {
                char name[48];
                snprintf(name, sizeof name, "htiny_32x32_%s", order_tag);
                if (try_pick(table, p, alignment, name, 1, kernel, split)) return;
            }
            // A shape hint (about half of the tile work, unequal tiles) is ranked like the general problem, with one
            // measured exception: when the 256 x 256 direct-to-LDS grid leaves compute units idle anyway, the
            // 128 x 128 tiles balance the unequal work better (3072: TRMM 59 against 77 us, SYRK 58 against 76)
            if (!f32 && p.shape != MG_SHAPE_GENERAL && best == 0 && !tried[2] &&
                ceil_div(p.m, 256) * ceil_div(p.n, 256) <= (kComputeUnits * 3) / 4)
                best = 2;
            // FP32 work-groups take turns on a compute unit, so unequal tiles (skipped ones, narrowed K ranges)
            // only pay off when a compute unit gets many of them: the small tiles win at every size measured
            // (SYRK 4096: 974 / 923 / 695 / 618 us from the 256 x 256 to the 64 x 64 tile, TRMM 950 / 614 / 596 / 541;
            // SYRK 8192: 4958 / 4690 / 5044 us on 128 x 128 / 128 x 64 / 64 x 64)
            // (a triangular operand beyond 6144 x 6144 outputs is ranked like the general problem: TRMM 8192 takes
            // 4342 us that way, 4723 us on 64 x 64 tiles)
            if (f32 && p.shape != MG_SHAPE_GENERAL &&
                (p.shape == MG_SHAPE_C_LOWER || p.shape == MG_SHAPE_C_UPPER || p.m * p.n <= int64_t(6144) * 6144)) {
                const bool c_shape = p.shape == MG_SHAPE_C_LOWER || p.shape == MG_SHAPE_C_UPPER;
                const int small = c_shape && p.m * p.n > int64_t(4096) * 4096 ? 3 : 4;
                if (!tried[small]) best = small;
                else if (!tried[7 - small]) best = 7 - small;
            }
            tried[best] = true;
            const TileChoice &tc = tiles[best];
            const int want = best_slices;
            // a factor whose last slice would be empty is illegal: take the next smaller one
            for (int w = want; w >= 1; --w)
                if (try_mfma(table, p, alignment, tc.tag, w, kernel, split)) return;
        }
    }
    try_pick(table, p, alignment, f32 ? "direct_f32_64x64x16" : "direct_f16_64x64x16", 1, kernel, split);
}

int32_t select_batched(const std::vector<KernelEntry> &table, const BatchedProblem &p)
{
    // one wavefront per instance while the instance fits the register blocks (<= 64 in every extent); with
    // more 16^3 instances than wavefronts fit on the chip at once (256 compute units x 32), two per wavefront:
    // measured 7.0 -> 6.4 us (FP32) and 5.3 -> 4.7 us (FP16) for 10000 instances, no gain from four, a loss
    // below ~4000 instances
    static const char *const few[] = {"batched_wave_16", "batched_wave_32", "batched_wave_64w1"};
    static const char *const many[] = {"batched_wave_16x2", "batched_wave_32", "batched_wave_64w1"};
    // (FP32 instances smaller than 16^3 take the bounds-checked flavour, which gains nothing from the second
    // instance: 10000 x 8^3 5.5 us one per wavefront, 5.9 us two)
    const bool whole16 = p.m == 16 && p.n == 16 && p.k == 16;
    // FP32 instances whose operands no longer fit the last-level cache by a wide margin (HBM-real calls) are faster one
    // per wavefront again; 16^3, us one / two per wavefront: 120000 instances (379 MB of operands) 82.3 / 79.5, 140000
    // (442 MB) 101.2 / 107.9, 160000 117.3 / 131.6, 200000 (631 MB) 145.6 / 162.7.  FP16 stays with two (320000 instances,
    // 505 MB: 141.0 / 122.5).
    const double operand_bytes = static_cast<double>(p.batch) * static_cast<double>(p.m * p.k + p.k * p.n + p.m * p.n) * (p.dtype == MG_F32 ? 4.0 : 2.0);
    const bool streams_from_hbm = p.dtype == MG_F32 && operand_bytes > 410.0e6;
    const char *const *tags = p.batch >= 32 * kComputeUnits && !streams_from_hbm &&
                              (p.dtype != MG_F32 || whole16 || p.m > 16 || p.n > 16 || p.k > 16) ? many : few;
    const char *prefix = p.dtype == MG_F32 ? "" : "h";
    const char *contig = p.a_trans ? (p.b_trans ? "kn" : "kk") : (p.b_trans ? "mn" : "mk");
    // whole 64^3 instances with A along m and B along k: the kernels whose lanes are rows of C ask for A, B and C in whole
    // adjacent columns (1 KB runs instead of 64-byte ones): FP32 10000 instances 155 -> 116 us, FP16 85 -> 49 us.  FP32 with
    // four wavefronts per instance (a quarter of the columns each) is never slower than one and faster for few
    // instances (us, one / four: 200 instances 8.9 / 6.0, 500: 9.8 / 7.8, 1000: 14.4 / 14.2, 4000: 43.3 / 41.6, 10000: 116.6 / 116.3)
    for (const char *name : {"batched_rows_64w4_mk_full", "batched_rows_64_mk_full", "hbatched_rows_64_mk_full"}) {
        const int32_t id = find(table, name);
        if (id >= 0 && table[id].legal_batched(p)) return id;
    }
    for (int t = 0; t < 3; ++t) {
        const char *tag = tags[t];
        char name[96];
        snprintf(name, sizeof name, "%s%s_%s_full", prefix, tag, contig);
        int32_t id = find(table, name);
        if (id >= 0 && table[id].legal_batched(p)) return id;
        snprintf(name, sizeof name, "%s%s_%s", prefix, tag, contig);
        id = find(table, name);
        if (id >= 0 && table[id].legal_batched(p)) return id;
    }
    const int32_t id = find(table, p.dtype == MG_F32 ? "batched_direct_f32_64x64x16" : "batched_direct_f16_64x64x16");
    if (id >= 0 && table[id].legal_batched(p)) return id;
    return -1;
}

}  // namespace mg

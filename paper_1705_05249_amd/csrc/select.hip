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
    snprintf(name, sizeof name, "%s_%s", tag, contig);
    if (try_pick(table, p, alignment, name, split, kernel, out_split)) return true;
    snprintf(name, sizeof name, "%s_%s_edge", tag, contig);
    return try_pick(table, p, alignment, name, split, kernel, out_split);
}

struct TileChoice {
    const char *tag;
    int bm, bn;
};

constexpr int kComputeUnits = 256;

}  // namespace

void select_config(const std::vector<KernelEntry> &table, const Problem &p, int64_t alignment, int32_t *kernel,
                   int32_t *split)
{
    *kernel = -1;
    *split = 1;
    const bool f32 = p.dtype == MG_F32;
    if (p.alpha == 0.f || p.k == 0) {
        try_pick(table, p, alignment, f32 ? "scale_f32" : "scale_f16", 1, kernel, split);
        return;
    }
    if (p.m >= 64 && p.n >= 64) {
        // largest macro tile that still gives most compute units a tile of their own
        static const TileChoice f16_tiles[] = {{"hmfma_256x256x64_w2x2", 256, 256}, {"hmfma_128x128x64_w2x2", 128, 128}};
        static const TileChoice f32_tiles[] = {{"smfma_128x128x32_w2x2", 128, 128}};
        const TileChoice *tiles = f32 ? f32_tiles : f16_tiles;
        const int count = f32 ? 1 : 2;
        for (int i = 0; i < count; ++i) {
            const int64_t n_tiles = ceil_div(p.m, tiles[i].bm) * ceil_div(p.n, tiles[i].bn);
            if (n_tiles >= (kComputeUnits * 3) / 4 || i == count - 1) {
                if (try_mfma(table, p, alignment, tiles[i].tag, 1, kernel, split)) return;
            }
        }
    }
    try_pick(table, p, alignment, f32 ? "direct_f32_64x64x16" : "direct_f16_64x64x16", 1, kernel, split);
}

int32_t select_batched(const std::vector<KernelEntry> &table, const BatchedProblem &p)
{
    // one wavefront per instance while the instance fits the register blocks (<= 64 in every extent)
    static const char *const tags[] = {"batched_wave_16", "batched_wave_32", "batched_wave_64"};
    const char *contig = p.a_trans ? (p.b_trans ? "kn" : "kk") : (p.b_trans ? "mn" : "mk");
    for (const char *tag : tags) {
        char name[96];
        snprintf(name, sizeof name, "%s_%s_full", tag, contig);
        int32_t id = find(table, name);
        if (id >= 0 && table[id].legal_batched(p)) return id;
        snprintf(name, sizeof name, "%s_%s", tag, contig);
        id = find(table, name);
        if (id >= 0 && table[id].legal_batched(p)) return id;
    }
    const int32_t id = find(table, "batched_direct_f32_64x64x16");
    if (id >= 0 && table[id].legal_batched(p)) return id;
    return -1;
}

}  // namespace mg

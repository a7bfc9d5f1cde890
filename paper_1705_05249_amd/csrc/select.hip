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
    try_pick(table, p, alignment, f32 ? "direct_f32_64x64x16" : "direct_f16_64x64x16", 1, kernel, split);
}

int32_t select_batched(const std::vector<KernelEntry> &table, const BatchedProblem &p)
{
    const int32_t id = find(table, "batched_direct_f32_64x64x16");
    if (id >= 0 && table[id].legal_batched(p)) return id;
    return -1;
}

}  // namespace mg

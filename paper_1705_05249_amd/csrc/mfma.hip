#include "internal.h"

namespace mg {
void register_mfma_f16_a(std::vector<KernelEntry> &table);
void register_mfma_f16_b(std::vector<KernelEntry> &table);
void register_mfma_f16_c(std::vector<KernelEntry> &table);
void register_mfma_f32_a(std::vector<KernelEntry> &table);

void register_mfma(std::vector<KernelEntry> &table)
{
    register_mfma_f16_a(table);
    register_mfma_f16_b(table);
    register_mfma_f16_c(table);
    register_mfma_f32_a(table);
}
}  // namespace mg

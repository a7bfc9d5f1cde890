// Registration order of the compiled MFMA tile configurations (one translation unit per tile shape).
#include "internal.h"

namespace mg {
void register_hmfma_256x256x64_w2x2(std::vector<KernelEntry> &table);
void register_hmfma_256x256x64_w2x4(std::vector<KernelEntry> &table);
void register_hmfma_256x128x64_w2x2(std::vector<KernelEntry> &table);
void register_hmfma_128x128x64_w2x2(std::vector<KernelEntry> &table);
void register_hmfma_128x64x64_w2x2(std::vector<KernelEntry> &table);
void register_hmfma_64x64x64_w2x2(std::vector<KernelEntry> &table);
void register_hdma16_256x256x64(std::vector<KernelEntry> &table);
void register_hdma16_small(std::vector<KernelEntry> &table);
void register_hpp16_256x256x64(std::vector<KernelEntry> &table);
void register_hclip(std::vector<KernelEntry> &table);
void register_tiny(std::vector<KernelEntry> &table);
void register_hdma_256x256x64_w2x2(std::vector<KernelEntry> &table);
void register_hdma_256x256x64_w2x4(std::vector<KernelEntry> &table);
void register_smfma_256x256x32_w2x2(std::vector<KernelEntry> &table);
void register_smfma_256x256x32_w2x4(std::vector<KernelEntry> &table);
void register_smfma_256x128x32_w4x2(std::vector<KernelEntry> &table);
void register_smfma_256x128x32_w2x2(std::vector<KernelEntry> &table);
void register_smfma_128x128x32_w2x2(std::vector<KernelEntry> &table);
void register_smfma_128x64x32_w2x2(std::vector<KernelEntry> &table);
void register_smfma_64x64x32_w2x2(std::vector<KernelEntry> &table);

void register_mfma(std::vector<KernelEntry> &table)
{
    register_hmfma_256x256x64_w2x2(table);
    register_hmfma_256x256x64_w2x4(table);
    register_hmfma_256x128x64_w2x2(table);
    register_hmfma_128x128x64_w2x2(table);
    register_hmfma_128x64x64_w2x2(table);
    register_hmfma_64x64x64_w2x2(table);
    register_hdma16_256x256x64(table);
    register_hdma16_small(table);
    register_hpp16_256x256x64(table);
    register_hclip(table);
    register_hdma_256x256x64_w2x2(table);
    register_hdma_256x256x64_w2x4(table);
    register_smfma_256x256x32_w2x2(table);
    register_smfma_256x256x32_w2x4(table);
    register_smfma_256x128x32_w4x2(table);
    register_smfma_256x128x32_w2x2(table);
    register_smfma_128x128x32_w2x2(table);
    register_smfma_128x64x32_w2x2(table);
    register_smfma_64x64x32_w2x2(table);
    register_tiny(table);
}
}  // namespace mg

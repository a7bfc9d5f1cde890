// Direct-to-LDS FP16 kernels on 16x16 MFMA blocks (both operands contiguous along k), tile 256 x 256 x 64.
#include "mfma_dma_host.h"
namespace mg {
void register_hdma16_256x256x64(std::vector<KernelEntry> &table)
{
    table.push_back(MfmaDmaConfig<256, 256, 2, 2, true, true, 16>::entry("hdma16_256x256x64_w2x2_kk"));
    table.push_back(MfmaDmaConfig<256, 256, 2, 4, true, true, 16>::entry("hdma16_256x256x64_w2x4_kk"));
}
}  // namespace mg

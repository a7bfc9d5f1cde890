// Direct-to-LDS FP16 kernels on 16x16 MFMA blocks, tile 256 x 256 x 64.
#include "mfma_dma_host.h"
namespace mg {
void register_hdma16_256x256x64(std::vector<KernelEntry> &table)
{
    table.push_back(MfmaDmaConfig<256, 256, 2, 2, true, true, 16>::entry("hdma16_256x256x64_w2x2_kk"));
    table.push_back(MfmaDmaConfig<256, 256, 2, 4, true, true, 16>::entry("hdma16_256x256x64_w2x4_kk"));
    table.push_back(MfmaDmaConfig<256, 256, 2, 4, false, true, 16>::entry("hdma16_256x256x64_w2x4_mk"));
    table.push_back(MfmaDmaConfig<256, 256, 2, 4, true, false, 16>::entry("hdma16_256x256x64_w2x4_kn"));
    table.push_back(MfmaDmaConfig<256, 256, 2, 4, false, false, 16>::entry("hdma16_256x256x64_w2x4_mn"));
}
}  // namespace mg

// Direct-to-LDS FP16 kernels on 16x16 MFMA blocks with smaller work-group tiles (256 x 128 and 128 x 128),
// for problems with too few 256 x 256 tiles to fill the chip.
#include "mfma_dma_host.h"
namespace mg {
void register_hdma16_small(std::vector<KernelEntry> &table)
{
    table.push_back(MfmaDmaConfig<256, 128, 4, 2, true, true, 16>::entry("hdma16_256x128x64_w4x2_kk"));
    table.push_back(MfmaDmaConfig<256, 128, 4, 2, false, true, 16>::entry("hdma16_256x128x64_w4x2_mk"));
    table.push_back(MfmaDmaConfig<256, 128, 4, 2, true, false, 16>::entry("hdma16_256x128x64_w4x2_kn"));
    table.push_back(MfmaDmaConfig<256, 128, 4, 2, false, false, 16>::entry("hdma16_256x128x64_w4x2_mn"));
    table.push_back(MfmaDmaConfig<128, 128, 2, 2, true, true, 16>::entry("hdma16_128x128x64_w2x2_kk"));
    table.push_back(MfmaDmaConfig<128, 128, 2, 2, false, true, 16>::entry("hdma16_128x128x64_w2x2_mk"));
    table.push_back(MfmaDmaConfig<128, 128, 2, 2, true, false, 16>::entry("hdma16_128x128x64_w2x2_kn"));
    table.push_back(MfmaDmaConfig<128, 128, 2, 2, false, false, 16>::entry("hdma16_128x128x64_w2x2_mn"));
}
}  // namespace mg

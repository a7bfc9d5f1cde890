// Direct-to-LDS FP16 kernels on 16x16 MFMA blocks with smaller work-group tiles (256 x 128 and 128 x 128),
// for problems with too few 256 x 256 tiles to fill the chip.  The 128 x 128 tile comes with four wavefronts of
// 64 x 64 and with eight of 64 x 32 (two per SIMD: 5-10 % faster when a compute unit holds a single work-group).
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
    table.push_back(MfmaDmaConfig<128, 128, 2, 4, true, true, 16>::entry("hdma16_128x128x64_w2x4_kk"));
    table.push_back(MfmaDmaConfig<128, 128, 2, 4, false, true, 16>::entry("hdma16_128x128x64_w2x4_mk"));
    table.push_back(MfmaDmaConfig<128, 128, 2, 4, true, false, 16>::entry("hdma16_128x128x64_w2x4_kn"));
    table.push_back(MfmaDmaConfig<128, 128, 2, 4, false, false, 16>::entry("hdma16_128x128x64_w2x4_mn"));
}
}  // namespace mg

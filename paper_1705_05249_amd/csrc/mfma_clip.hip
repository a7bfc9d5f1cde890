// The direct-to-LDS FP16 kernels for operands padded to whole tiles in a workspace and the caller's own C: tiles
// 256 x 256 x 64 and 128 x 128 x 64 on eight wavefronts, bounds-checked epilogue (names: ...c_...).
#include "mfma_dma_host.h"
namespace mg {
void register_hclip(std::vector<KernelEntry> &table)
{
    table.push_back(MfmaPpConfig<false, true>::entry("hpp16c_256x256x64_w2x4_mk"));
    table.push_back(MfmaPpConfig<true, true>::entry("hpp16c_256x256x64_w2x4_kk"));
    table.push_back(MfmaDmaConfig<256, 256, 2, 4, true, false, 16, true>::entry("hdma16c_256x256x64_w2x4_kn"));
    table.push_back(MfmaDmaConfig<256, 256, 2, 4, false, false, 16, true>::entry("hdma16c_256x256x64_w2x4_mn"));
    table.push_back(MfmaDmaConfig<128, 128, 2, 4, true, true, 16, true>::entry("hdma16c_128x128x64_w2x4_kk"));
    table.push_back(MfmaDmaConfig<128, 128, 2, 4, false, true, 16, true>::entry("hdma16c_128x128x64_w2x4_mk"));
    table.push_back(MfmaDmaConfig<128, 128, 2, 4, true, false, 16, true>::entry("hdma16c_128x128x64_w2x4_kn"));
    table.push_back(MfmaDmaConfig<128, 128, 2, 4, false, false, 16, true>::entry("hdma16c_128x128x64_w2x4_mn"));
}
}  // namespace mg

// The 256 x 256 x 64 FP16 kernels for operands padded to whole tiles in a workspace and the caller's own C:
// direct-to-LDS loads, bounds-checked epilogue (names: ...c_...).
#include "mfma_dma_host.h"
namespace mg {
void register_hclip_256x256x64(std::vector<KernelEntry> &table)
{
    table.push_back(MfmaPpConfig<false, true>::entry("hpp16c_256x256x64_w2x4_mk"));
    table.push_back(MfmaPpConfig<true, true>::entry("hpp16c_256x256x64_w2x4_kk"));
    table.push_back(MfmaDmaConfig<256, 256, 2, 4, true, false, 16, true>::entry("hdma16c_256x256x64_w2x4_kn"));
    table.push_back(MfmaDmaConfig<256, 256, 2, 4, false, false, 16, true>::entry("hdma16c_256x256x64_w2x4_mn"));
}
}  // namespace mg

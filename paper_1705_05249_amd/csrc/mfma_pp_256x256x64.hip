// FP16 kernels whose wavefronts take turns between LDS reads and MFMAs, tile 256 x 256 x 64.
#include "mfma_dma_host.h"
namespace mg {
void register_hpp16_256x256x64(std::vector<KernelEntry> &table)
{
    table.push_back(MfmaPpConfig<false>::entry("hpp16_256x256x64_w2x4_mk"));
    table.push_back(MfmaPpConfig<true>::entry("hpp16_256x256x64_w2x4_kk"));
}
}  // namespace mg

// Direct-to-LDS FP16 kernels, tile 256 x 256 x 64, 2 x 4 wavefronts.
#include "mfma_dma_host.h"
namespace mg {
void register_hdma_256x256x64_w2x4(std::vector<KernelEntry> &table)
{
    MG_DMA_REGISTER(table, "hdma_256x256x64_w2x4", 256, 256, 2, 4)
}
}  // namespace mg

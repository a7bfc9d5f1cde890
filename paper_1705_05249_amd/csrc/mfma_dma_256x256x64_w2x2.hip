// Direct-to-LDS FP16 kernels, tile 256 x 256 x 64, 2 x 2 wavefronts.
#include "mfma_dma_host.h"
namespace mg {
void register_hdma_256x256x64_w2x2(std::vector<KernelEntry> &table)
{
    MG_DMA_REGISTER(table, "hdma_256x256x64_w2x2", 256, 256, 2, 2)
}
}  // namespace mg

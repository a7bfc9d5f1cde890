// MFMA macro-tile kernels, tile 256 x 256 x 32, 2 x 2 wavefronts, f32 storage.
#include "mfma_host.h"
namespace mg {
void register_smfma_256x256x32_w2x2(std::vector<KernelEntry> &table)
{
    MG_MFMA_REGISTER_WHOLE(table, float, "smfma_256x256x32_w2x2", 256, 256, 32, 2, 2)
}
}  // namespace mg

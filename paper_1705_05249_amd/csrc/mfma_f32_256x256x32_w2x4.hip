// MFMA macro-tile kernels, tile 256 x 256 x 32, 2 x 4 wavefronts (two per SIMD), f32 storage.
#include "mfma_host.h"
namespace mg {
void register_smfma_256x256x32_w2x4(std::vector<KernelEntry> &table)
{
    MG_MFMA_REGISTER(table, float, "smfma_256x256x32_w2x4", 256, 256, 32, 2, 4)
}
}  // namespace mg

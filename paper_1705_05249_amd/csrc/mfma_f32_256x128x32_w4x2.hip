// MFMA macro-tile kernels, tile 256 x 128 x 32, 4 x 2 wavefronts (two per SIMD), f32 storage.
#include "mfma_host.h"
namespace mg {
void register_smfma_256x128x32_w4x2(std::vector<KernelEntry> &table)
{
    MG_MFMA_REGISTER(table, float, "smfma_256x128x32_w4x2", 256, 128, 32, 4, 2)
}
}  // namespace mg

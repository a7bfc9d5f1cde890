// MFMA macro-tile kernels, tile 256 x 256 x 64, 2 x 4 wavefronts, f16 storage.
#include "mfma_host.h"
namespace mg {
void register_hmfma_256x256x64_w2x4(std::vector<KernelEntry> &table)
{
    MG_MFMA_REGISTER(table, _Float16, "hmfma_256x256x64_w2x4", 256, 256, 64, 2, 4)
}
}  // namespace mg

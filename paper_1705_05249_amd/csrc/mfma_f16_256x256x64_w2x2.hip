// MFMA macro-tile kernels, tile 256 x 256 x 64, 2 x 2 wavefronts, f16 storage.
#include "mfma_host.h"
namespace mg {
void register_hmfma_256x256x64_w2x2(std::vector<KernelEntry> &table)
{
    MG_MFMA_REGISTER_WHOLE(table, _Float16, "hmfma_256x256x64_w2x2", 256, 256, 64, 2, 2)
}
}  // namespace mg

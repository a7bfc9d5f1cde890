// MFMA macro-tile kernels, tile 128 x 64 x 64, 2 x 2 wavefronts, f16 storage.
#include "mfma_host.h"
namespace mg {
void register_hmfma_128x64x64_w2x2(std::vector<KernelEntry> &table)
{
    MG_MFMA_REGISTER(table, _Float16, "hmfma_128x64x64_w2x2", 128, 64, 64, 2, 2)
}
}  // namespace mg

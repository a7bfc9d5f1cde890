// MFMA macro-tile kernels, tile 64 x 64 x 32, 2 x 2 wavefronts, f32 storage.
#include "mfma_host.h"
namespace mg {
void register_smfma_64x64x32_w2x2(std::vector<KernelEntry> &table)
{
    MG_MFMA_REGISTER(table, float, "smfma_64x64x32_w2x2", 64, 64, 32, 2, 2)
    // the bounds-checked "mk" kernel fed from an image instead of a stored column matrix (convolution without the
    // unfold pass)
    table.push_back(MfmaConfig<float, 64, 64, 32, 2, 2, false, true, true, 32, true>::entry("sconv_64x64x32_w2x2"));
}
}  // namespace mg

// MFMA macro-tile kernels, tile 64 x 64 x 64, 2 x 2 wavefronts, f16 storage.
#include "mfma_host.h"
namespace mg {
void register_hmfma_64x64x64_w2x2(std::vector<KernelEntry> &table)
{
    MG_MFMA_REGISTER(table, _Float16, "hmfma_64x64x64_w2x2", 64, 64, 64, 2, 2)
    // the bounds-checked "mk" kernel fed from an image instead of a stored column matrix (convolution without the
    // unfold pass)
    table.push_back(MfmaConfig<_Float16, 64, 64, 64, 2, 2, false, true, true, 32, true>::entry("hconv_64x64x64_w2x2"));
}
}  // namespace mg

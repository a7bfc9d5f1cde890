#include "mfma_host.h"
namespace mg {
void register_mfma_f16_c(std::vector<KernelEntry> &table)
{
    MG_MFMA_REGISTER(table, _Float16, "hmfma_256x256x64_w2x4", 256, 256, 64, 2, 4)
}
}  // namespace mg

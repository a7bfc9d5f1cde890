#include "mfma_host.h"
namespace mg {
void register_mfma_f16_b(std::vector<KernelEntry> &table)
{
    MG_MFMA_REGISTER(table, _Float16, "hmfma_128x128x64_w2x2", 128, 128, 64, 2, 2)
}
}  // namespace mg

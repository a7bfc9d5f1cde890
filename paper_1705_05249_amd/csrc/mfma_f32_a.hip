#include "mfma_host.h"
namespace mg {
void register_mfma_f32_a(std::vector<KernelEntry> &table)
{
    MG_MFMA_REGISTER(table, float, "smfma_128x128x32_w2x2", 128, 128, 32, 2, 2)
}
}  // namespace mg

// Placeholder until the MFMA kernel lands: nothing is supported yet.
#include "yoco_common.h"
namespace yoco {
bool swa_mfma_supported(const AttnView&, int) { return false; }
hipError_t launch_swa_mfma(const AttnView&, hipStream_t) { return hipErrorNotSupported; }
}  // namespace yoco

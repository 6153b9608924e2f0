// Placeholder until the streaming decode kernel lands: nothing is supported yet.
#include "yoco_common.h"
namespace yoco {
bool decode_bf16_supported(const yoco_kv_cache&, int) { return false; }
hipError_t launch_decode_bf16(const yoco_kv_cache&, const void*, const int64_t*, int, float, float*, int, hipStream_t) {
  return hipErrorNotSupported;
}
}  // namespace yoco

// Chunkwise gated retention on the matrix cores (section 3.1, Eq. 6). Placeholder: no shape is supported yet.
#include "yoco_common.h"

namespace yoco {

bool gret_chunk_supported(int, int64_t, int, int, int, int, int) { return false; }
size_t gret_chunk_workspace(int, int64_t, int, int) { return 0; }
hipError_t launch_gret_chunk(const GretView&, int, void*, hipStream_t) { return hipErrorNotSupported; }

}  // namespace yoco

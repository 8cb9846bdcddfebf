// Decode attention over the MXFP4 cache (Sec. IV-D(2)) -- placeholder until the kernel lands.
#include "bd_common.h"

namespace bd {
hipError_t launch_decode_mx(const bd_cache*, const void*, int, float, int, float*, float*, hipStream_t) {
  return hipErrorNotSupported;
}
}  // namespace bd

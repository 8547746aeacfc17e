#include "common.h"
namespace nsa {
hipError_t launch_bwd(const Problem&, const IndexLayout&, const void*, const void*, const void*, const void*,
                      const float*, const void*, const void*, void*, float*, float*, void*, void*, void*,
                      hipStream_t) {
  return hipErrorNotSupported;
}
}  // namespace nsa

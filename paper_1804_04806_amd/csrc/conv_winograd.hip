// Winograd F(2x2,3x3) -- placeholder until the kernels land: reports "does not apply".
#include "kernels.h"

namespace ucd {
bool winograd_applies(const Dims &, int) { return false; }
size_t winograd_ws_bytes(const Dims &, int, int) { return (size_t)-1; }
hipError_t winograd_fwd(const Dims &, int, const float *, const float *, float *, float *, hipStream_t)
{
    return hipErrorNotSupported;
}
hipError_t winograd_bwd_data(const Dims &, int, const float *, const float *, float *, float *, hipStream_t)
{
    return hipErrorNotSupported;
}
}  // namespace ucd

#include "xnor_internal.hpp"
namespace xnor {
bool conv_tiled_supports(const Geom &) { return false; }
hipError_t launch_conv_tiled(const uint32_t *, const uint32_t *, const float *, const float *,
                             const Geom &, float *, int32_t *, hipStream_t) { return hipErrorNotSupported; }
}

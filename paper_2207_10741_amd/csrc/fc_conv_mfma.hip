#include "fc_internal.hpp"
namespace fc {
bool conv_mfma_supported(const Geom &, int, int) { return false; }
hipError_t launch_conv_mfma(const Geom &, int, int, const void *, const uint8_t *, const void *, const float *,
                            const int32_t *, const int32_t *, void *, hipStream_t)
{
    return hipErrorNotSupported;
}
} // namespace fc

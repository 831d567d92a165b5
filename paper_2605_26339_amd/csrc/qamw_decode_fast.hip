// Shape-specialised decoder (placeholder: not yet enabled).
#include "qamw_common.hpp"
#include "qamw_internal.hpp"
namespace qamw {
bool fast_decode_supported(const Problem &) { return false; }
hipError_t launch_decode_fast(const uint8_t *, const float *, const Problem &, void *, int64_t, bool) {
    return hipErrorNotSupported;
}
}  // namespace qamw

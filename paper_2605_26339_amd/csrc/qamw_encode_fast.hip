// Shape-specialised encoder (placeholder: not yet enabled).
#include "qamw_common.hpp"
#include "qamw_internal.hpp"
namespace qamw {
bool fast_encode_supported(const Problem &) { return false; }
hipError_t launch_encode_fast(const void *, int, int64_t, const Problem &, const float *, uint8_t *) {
    return hipErrorNotSupported;
}
}  // namespace qamw

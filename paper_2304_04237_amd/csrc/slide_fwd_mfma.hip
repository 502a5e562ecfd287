// placeholder, replaced by the matrix-core forward
#include "slide_internal.h"
namespace slide {
bool fwd_mfma_supported(const Problem&) { return false; }
hipError_t launch_fwd_mfma(const Problem&, const void*, const void*, const void*, const float*,
                           const float*, const float*, void*, hipStream_t) { return hipErrorNotSupported; }
}

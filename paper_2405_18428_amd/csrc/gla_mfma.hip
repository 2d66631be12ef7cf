// placeholder until the MFMA engine lands
#include "gla_common.h"
namespace gla {
bool mfma_engine_supports(const Params &) { return false; }
hipError_t launch_mfma_span(const Params &, SpanMode, hipStream_t) { return hipErrorNotSupported; }
}  // namespace gla

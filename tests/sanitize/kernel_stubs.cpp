// Stand-ins for the device side of the library in the sanitizer build of its host code: the
// host-only tests never launch anything, so every launch answers "not supported".
#include "taper_internal.h"

namespace taper {
hipError_t static_scratch(int, void**) { return hipErrorNotSupported; }
hipError_t launch_zero_words(int32_t*, int64_t, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_decode(const StepArgs&, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_kv_append(const void*, const void*, const int64_t*, void*, int, int, int, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_stream_read(const void*, int64_t, int, unsigned*, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_resolve_slots(const StepArgs&, int64_t*, int64_t, hipStream_t) { return hipErrorNotSupported; }
}  // namespace taper

#include <hip/hip_runtime.h>
#include "igemm.h"
namespace glowmi {
bool deep_i8_applicable(const Problem&) { return false; }
hipError_t launch_deep_i8(const Problem&, hipStream_t, const char**) { return hipErrorNotSupported; }
}

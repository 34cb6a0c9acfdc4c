#include <hip/hip_runtime.h>
#include "igemm.h"
namespace glowmi {
bool fc_small_f32_applicable(const Problem&) { return false; }
hipError_t launch_fc_small_f32(const Problem&, hipStream_t, const char**) { return hipErrorNotSupported; }
}

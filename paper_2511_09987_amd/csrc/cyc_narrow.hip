// placeholder until the streaming kernel lands
#include "cyc_internal.h"
namespace cyc {
bool supports_narrow(const Problem &) { return false; }
hipError_t launch_narrow(const Problem &, hipStream_t) { return hipErrorInvalidValue; }
}

// placeholder until the stem kernel lands
#include "cvx_device.h"
namespace cvx {
bool stem_supported(const ConvArgs&, const char**) { return false; }
hipError_t launch_stem(const ConvArgs&, hipStream_t) { return hipErrorNotSupported; }
}

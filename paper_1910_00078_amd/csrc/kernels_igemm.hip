// placeholder until the MFMA kernel lands
#include "cvx_device.h"
namespace cvx {
bool igemm_supported(const ConvArgs&, const char**) { return false; }
hipError_t launch_igemm(const ConvArgs&, hipStream_t) { return hipErrorNotSupported; }
}

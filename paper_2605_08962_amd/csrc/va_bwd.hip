#include "va_device.h"
#include "va_internal.h"
namespace va {
hipError_t launch_bwd_delta(const BwdArgs&, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_bwd_dkdv(const BwdArgs&, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_bwd_dq(const BwdArgs&, hipStream_t) { return hipErrorNotSupported; }
}

#include "kernels.h"
namespace va {
hipError_t launch_fwd_fp8(const AttnParams&, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_bwd_delta(const AttnParams&, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_bwd_dkdv(const AttnParams&, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_bwd_dq(const AttnParams&, hipStream_t) { return hipErrorNotSupported; }
}

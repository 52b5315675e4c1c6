// FP8 (E4M3) forward: placeholder until the kernel lands.
#include "kernels.h"
namespace va {
hipError_t launch_fwd_fp8(const AttnParams&, hipStream_t) { return hipErrorNotSupported; }
}

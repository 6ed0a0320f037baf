#include "common.h"
namespace bamboo {
hipError_t launch_attention_fwd_mfma(hipStream_t, const AttnDesc&) { return hipErrorNotSupported; }
hipError_t launch_attention_bwd_mfma(hipStream_t, const AttnDesc&) { return hipErrorNotSupported; }
}

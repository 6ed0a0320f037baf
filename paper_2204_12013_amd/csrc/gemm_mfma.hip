#include "common.h"
namespace bamboo {
hipError_t launch_gemm_mfma(hipStream_t, const GemmDesc&) { return hipErrorNotSupported; }
}

// placeholder, replaced below
#include "common.h"
namespace mslt {
bool gemm_mfma_supported(const GemmDesc&) { return false; }
hipError_t gemm_mfma(const GemmDesc&, int, float*, hipStream_t) { return hipErrorNotSupported; }
}

// placeholder, replaced below
#include "common.h"
namespace mslt {
bool attention_mfma_supported(int, int) { return false; }
hipError_t attention_fwd_mfma(const AttnDesc&, hipStream_t) { return hipErrorNotSupported; }
hipError_t attention_bwd_mfma(const AttnBwdDesc&, hipStream_t) { return hipErrorNotSupported; }
}

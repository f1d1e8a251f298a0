// placeholder until the MFMA attention lands
#include "common.h"
namespace stg {
bool attn_mfma_supported(const AttnArgs&) { return false; }
hipError_t attn_fwd_mfma(const AttnArgs&, hipStream_t) { return hipErrorNotSupported; }
hipError_t attn_bwd_mfma(const AttnArgs&, hipStream_t) { return hipErrorNotSupported; }
}

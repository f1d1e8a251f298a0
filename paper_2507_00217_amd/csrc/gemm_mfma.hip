// placeholder until the MFMA GEMM lands
#include "common.h"
namespace stg {
bool gemm_mfma_supported(const GemmArgs&) { return false; }
hipError_t gemm_mfma(const GemmArgs&, hipStream_t) { return hipErrorNotSupported; }
}

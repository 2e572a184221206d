// placeholder until the MFMA GEMM lands
#include "launch.h"
namespace sbp {
bool gemm_mfma_eligible(const GemmArgs&) { return false; }
hipError_t gemm_mfma(const GemmArgs&, hipStream_t) { return hipErrorNotSupported; }
}

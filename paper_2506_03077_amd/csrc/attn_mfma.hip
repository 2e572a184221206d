// placeholder until the MFMA attention lands
#include "launch.h"
namespace sbp {
bool attn_mfma_eligible(int, int, int, int) { return false; }
hipError_t attn_forward_mfma(const AttnArgs&, hipStream_t) { return hipErrorNotSupported; }
hipError_t attn_backward_mfma(const AttnArgs&, hipStream_t) { return hipErrorNotSupported; }
}

// bf16 MFMA kernels of the expert MLP - placeholder until the MFMA family lands: nothing is supported yet,
// so every call takes the float32-ALU kernels.
#include "xmoe_ffn.h"

namespace xmoe {
bool ffn_mfma_supported(const FfnArgs&) { return false; }
int ffn_fwd_mfma(const FfnArgs&, hipStream_t) { return XMOE_ERR_UNSUPPORTED; }
int ffn_bwd_mfma(const FfnArgs&, hipStream_t) { return XMOE_ERR_UNSUPPORTED; }
}  // namespace xmoe

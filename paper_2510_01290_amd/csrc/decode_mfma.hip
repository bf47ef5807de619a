// placeholder until the MFMA kernel lands
#include "decode_common.h"
namespace thinkv {
int decode_mfma_supported(const thinkv_config&) { return 0; }
int launch_decode_mfma(const thinkv_view&, const DecodeArgs&, hipStream_t) { return THINKV_E_UNSUPPORTED; }
}  // namespace thinkv

// Decode attention on the matrix cores: the kernel of thinkv_decode_attention (templates in
// decode_mfma_kernel.h; the variant that also leaves the pooled scores for the sparsity
// statistic is instantiated in decode_mfma_stat.hip, so the two compile side by side).
#include "decode_mfma_kernel.h"

namespace thinkv {

int decode_mfma_supported(const thinkv_config& c) {
  const int G = c.n_q_heads / c.n_kv_heads;
  return (c.head_dim == 64 || c.head_dim == 128) && G >= 1 && G <= 8;
}

int launch_decode_mfma(const thinkv_view& v, const DecodeArgs& a, hipStream_t st) { return launch_decode_mfma_t<false>(v, a, st); }

}  // namespace thinkv

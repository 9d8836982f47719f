// Fused MFMA path (placeholder until the kernels land): reports every problem as unsupported,
// so DARK_PATH_AUTO uses the fp32 kernels and DARK_PATH_FUSED fails loudly.
#include "common.h"

namespace dark {
bool fused_supported(const Problem&, int, bool) { return false; }
dark_status fused_attn_fwd(const Problem&, Arena&, const void*, const void*, const void*, const float*,
                           const float*, void*) {
  return DARK_EUNSUPPORTED;
}
dark_status fused_attn_causal_fwd(const Problem&, Arena&, const void*, const void*, const void*, const float*,
                                  const float*, void*) {
  return DARK_EUNSUPPORTED;
}
}  // namespace dark

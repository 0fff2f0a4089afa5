// bfloat16 MFMA tree-attention kernel (placeholder until the kernel lands: nothing is routed here).
#include "attn_common.h"

namespace hs {
bool attn_mfma_supported(int D, hs_dtype dt) {
  (void)D;
  (void)dt;
  return false;
}
hs_status attn_mfma_launch(const AttnArgs&, const int32_t*, const int64_t*, hipStream_t) {
  return fail(HS_ERR_UNSUPPORTED, "MFMA tree attention is not built");
}
}  // namespace hs

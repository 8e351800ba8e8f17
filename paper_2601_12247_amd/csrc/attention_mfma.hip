// bf16 non-causal attention on the MFMA matrix cores (placeholder until the kernel lands).
#include "common.h"
namespace pvf {
bool attention_mfma_supported(int, int, int) { return false; }
pvf_status launch_attention_mfma(pvf_ctx *ctx, hipStream_t, const void *, void *, int, int, int, int) {
  set_error(ctx, "attention_mfma: not built");
  return PVF_ENOTIMPL;
}
}  // namespace pvf

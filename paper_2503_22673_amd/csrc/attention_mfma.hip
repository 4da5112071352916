// MFMA flash-style attention kernels (bf16).  Placeholder translation unit:
// until the kernels are in, every shape is routed to the plain kernels.
#include "common.h"

bool attention_mfma_ok(const AttnParams& p) { (void)p; return false; }
int launch_attention_fwd_mfma(as_ctx* ctx, const AttnParams& p, hipStream_t st) {
  (void)p; (void)st; return as_fail(ctx, AS_ERR_SHAPE, "attention: MFMA kernel not available");
}
int launch_attention_bwd_mfma(as_ctx* ctx, const AttnParams& p, hipStream_t st) {
  (void)p; (void)st; return as_fail(ctx, AS_ERR_SHAPE, "attention: MFMA kernel not available");
}

// Encoder instantiations for the token norm over all kv heads (App. "Fused Hadamard-Norm
// Kernel").  -ffp-contract=off, as for every user of the encoder header.
//
// Two launches: oscar_token_norm_kernel computes the norms of the new tokens that go into
// pages (it reads every head of a token once), then the encoder kernel runs as usual and
// takes those norms from the pages' norm slots.  A single-token decode append never moves a
// new token into a page (a deferred flush holds residual tokens only), so it skips the first
// launch; tokens that stay in the residual window get their norm inside the encoder kernel.
#include "oscar_append_kernel.h"

int oscar_launch_append_all_heads(const AppendParams& P, dim3 grid, hipStream_t st) {
  const bool eager = (P.flags & OSCAR_APPEND_EAGER) != 0;
  if (P.T > 1 || eager) {
    switch (P.c.cfg.io_dtype) {
      case OSCAR_F32: launch_token_norms<float>(P, st); break;
      case OSCAR_BF16: launch_token_norms<__hip_bfloat16>(P, st); break;
      case OSCAR_F16: launch_token_norms<__half>(P, st); break;
      default: return OSCAR_ERR_UNSUPPORTED;
    }
  }
  return launch_append<XF_ALL_HEADS>(P, grid, st);
}

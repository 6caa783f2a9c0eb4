/* The public header must be plain C: compiled with a C compiler in the CPU test suite, and linked against
 * the shared library to prove that every declared entry point resolves.  No device is touched: the only
 * calls made are the ones that need none. */
#include <stdio.h>
#include "../include/flashdp.h"

int main(void) {
  /* take the address of every entry point so that the link fails if one is missing */
  typedef void (*fn_t)(void);
  fn_t syms[] = {
      (fn_t)flashdp_linear_dp_grad, (fn_t)flashdp_block_dp_grad, (fn_t)flashdp_block_dp_grad_micro,
      (fn_t)flashdp_workspace_bytes, (fn_t)flashdp_workspace_bytes_chunked, (fn_t)flashdp_last_chunk, (fn_t)flashdp_linear_dp_grad_static, (fn_t)flashdp_static_scratch_bytes, (fn_t)flashdp_plain_grad, (fn_t)flashdp_plain_grad_balanced, (fn_t)flashdp_plain_grad_balanced_workspace_bytes, (fn_t)flashdp_noise_field, (fn_t)flashdp_box_muller, (fn_t)flashdp_mfma_probe, (fn_t)flashdp_contraction_timeline,
      (fn_t)flashdp_set_stream, (fn_t)flashdp_set_workspace, (fn_t)flashdp_set_dtype, (fn_t)flashdp_set_layer,
      (fn_t)flashdp_set_schedule, (fn_t)flashdp_set_stages, (fn_t)flashdp_release, (fn_t)flashdp_last_schedule, (fn_t)flashdp_last_kernel,
      (fn_t)flashdp_status_string, (fn_t)flashdp_version};
  flashdp_layer_t L = {0};
  L.d_in = 5120; L.d_out = 13824; L.C = 1.0f; L.sigma = 1.0f;
  size_t need = flashdp_workspace_bytes(&L, 1, 8, 2048, FLASHDP_BF16, FLASHDP_SCHEDULE_SCRATCH);
  printf("%d %s %zu %zu\n", flashdp_version(), flashdp_status_string(FLASHDP_WORKSPACE_TOO_SMALL), need, sizeof(syms) / sizeof(syms[0]));
  return (need >= (size_t)8 * 5120 * 13824 * 2 && flashdp_linear_dp_grad(0, 0, 1, 1, 8, 8, 1.0f, 0.0f, 0, 0, 0) == FLASHDP_INVALID_ARGUMENT) ? 0 : 1;
}

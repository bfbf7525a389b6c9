// bf16 MFMA GEMM, operand layout "mn": A row-contiguous, B row-contiguous
// (one translation unit per layout so that the four compile in parallel).
#include "gemm_bf16_impl.h"

int stp_launch_gemm_bf16_mn(stp_ctx *ctx, const stp_gemm_args *a, hipStream_t s) {
  return launch_layout<false, false>(ctx, a, s);
}

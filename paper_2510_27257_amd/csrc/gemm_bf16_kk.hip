// bf16 MFMA GEMM, operand layout "kk": A k-contiguous, B k-contiguous
// (one translation unit per layout so that the four compile in parallel).
#include "gemm_bf16_impl.h"

int stp_launch_gemm_bf16_kk(stp_ctx *ctx, const stp_gemm_args *a, hipStream_t s) {
  return launch_layout<true, true>(ctx, a, s);
}

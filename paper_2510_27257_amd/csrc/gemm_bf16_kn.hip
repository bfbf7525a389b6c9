// bf16 MFMA GEMM, operand layout "kn": A k-contiguous, B row-contiguous
// (one translation unit per layout so that the four compile in parallel).
#include "gemm_bf16_impl.h"

int stp_launch_gemm_bf16_kn(stp_ctx *ctx, const stp_gemm_args *a, hipStream_t s) {
  return launch_layout<true, false>(ctx, a, s);
}

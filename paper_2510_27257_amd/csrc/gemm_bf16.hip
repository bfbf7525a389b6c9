// Dispatch of the bf16 MFMA GEMM to the translation unit built for the operand layout.
#include "common.h"

int stp_launch_gemm_bf16_kk(stp_ctx *ctx, const stp_gemm_args *a, hipStream_t s);
int stp_launch_gemm_bf16_kn(stp_ctx *ctx, const stp_gemm_args *a, hipStream_t s);
int stp_launch_gemm_bf16_mk(stp_ctx *ctx, const stp_gemm_args *a, hipStream_t s);
int stp_launch_gemm_bf16_mn(stp_ctx *ctx, const stp_gemm_args *a, hipStream_t s);

int stp_launch_gemm_bf16(stp_ctx *ctx, const stp_gemm_args *a, hipStream_t s) {
  const bool a_kc = !a->a_trans, b_kc = a->b_trans != 0;
  if (a_kc && b_kc) return stp_launch_gemm_bf16_kk(ctx, a, s);
  if (a_kc && !b_kc) return stp_launch_gemm_bf16_kn(ctx, a, s);
  if (!a_kc && b_kc) return stp_launch_gemm_bf16_mk(ctx, a, s);
  return stp_launch_gemm_bf16_mn(ctx, a, s);
}

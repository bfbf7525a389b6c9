// fp32 GEMM for the fp32 configuration (the tiny correctness workload): plain FMA
// arithmetic in true fp32 (no reduced-precision matrix mode), 64x64x16 LDS tiles,
// 4x4 outputs per thread, arbitrary operand strides so one kernel serves the
// forward, activation-gradient and weight-gradient forms.  Not a performance path.
#include "common.h"

namespace {
constexpr int TB = 64, TK = 16;

struct EpiF {
  float *C; int ldc; int accum;
  const float *bias; float bias_scale;
  const float *resid; int ldr; float resid_scale;
  int mode; float *C2; const float *aux; int ld2;
};

__global__ __launch_bounds__(256) void gemm_f32_kernel(const float *__restrict__ A, long sam, long sak,
                                                       const float *__restrict__ B, long sbk, long sbn, int M, int N,
                                                       int K, EpiF ep) {
  __shared__ float As[TK][TB + 1], Bs[TK][TB + 1];
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  const int m0 = blockIdx.y * TB, n0 = blockIdx.x * TB;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += TK) {
    for (int q = tid; q < TB * TK; q += 256) {
      int r, k;
      if (sak == 1) { k = q % TK; r = q / TK; } else { r = q % TB; k = q / TB; }
      As[k][r] = (m0 + r < M && k0 + k < K) ? A[(long)(m0 + r) * sam + (long)(k0 + k) * sak] : 0.f;
    }
    for (int q = tid; q < TB * TK; q += 256) {
      int c, k;
      if (sbk == 1) { k = q % TK; c = q / TK; } else { c = q % TB; k = q / TB; }
      Bs[k][c] = (n0 + c < N && k0 + k < K) ? B[(long)(k0 + k) * sbk + (long)(n0 + c) * sbn] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < TK; k++) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; i++) { a[i] = As[k][ty + 16 * i]; b[i] = Bs[k][tx + 16 * i]; }
#pragma unroll
      for (int i = 0; i < 4; i++)
#pragma unroll
        for (int j = 0; j < 4; j++) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; i++) {
    int row = m0 + ty + 16 * i;
    if (row >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; j++) {
      int col = n0 + tx + 16 * j;
      if (col >= N) continue;
      float val = acc[i][j];
      if (ep.bias) val += ep.bias[col] * ep.bias_scale;
      if (ep.resid) val += ep.resid[(size_t)row * ep.ldr + col] * ep.resid_scale;
      if (ep.accum) {
        ep.C[(size_t)row * ep.ldc + col] += val;
      } else {
        if (ep.mode == 2) val *= gelu_grad_f(ep.aux[(size_t)row * ep.ld2 + col]);
        ep.C[(size_t)row * ep.ldc + col] = val;
        if (ep.mode == 1) ep.C2[(size_t)row * ep.ld2 + col] = gelu_f(val);
      }
    }
  }
}
}  // namespace

int stp_launch_gemm_f32(stp_ctx *ctx, const stp_gemm_args *a, hipStream_t s) {
  EpiF ep;
  ep.C = (float *)a->C; ep.ldc = a->ldc; ep.accum = a->c_f32_accum;
  ep.bias = (const float *)a->bias; ep.bias_scale = a->bias_scale;
  ep.resid = (const float *)a->resid; ep.ldr = a->ldr; ep.resid_scale = a->resid_scale;
  ep.mode = a->epilogue; ep.C2 = (float *)a->C2; ep.aux = (const float *)a->aux; ep.ld2 = a->ld2;
  long sam = a->a_trans ? 1 : a->lda, sak = a->a_trans ? a->lda : 1;
  long sbk = a->b_trans ? 1 : a->ldb, sbn = a->b_trans ? a->ldb : 1;
  dim3 grid((a->N + TB - 1) / TB, (a->M + TB - 1) / TB), block(256);
  hipLaunchKernelGGL(gemm_f32_kernel, grid, block, 0, s, (const float *)a->A, sam, sak, (const float *)a->B, sbk, sbn,
                     a->M, a->N, a->K, ep);
  STP_LAUNCH_CHECK(ctx);
  return STP_OK;
}

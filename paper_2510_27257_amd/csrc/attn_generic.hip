// Plain attention forward / backward for the fp32 configuration: one 64-lane wave
// per (sequence, head, row); lanes split the head dimension (d <= 128) and every
// query-key dot product is a wave reduction.  True fp32 arithmetic throughout.
// This is the correctness path of the tiny workload, not a performance path; the
// bf16 workloads use the MFMA kernels.
// Grouped-query attention: nk key / value heads, query head i uses key / value head i / (n / nk); a row of
// qkv is [n Q heads | nk K heads | nk V heads].
#include "common.h"

int stp_launch_rowdot(stp_ctx *ctx, const stp_layer_desc *d, const void *a, const void *b, float *delta, hipStream_t s);

namespace {

template <typename T>
__global__ __launch_bounds__(256) void attn_fwd_generic(const T *__restrict__ qkv, T *__restrict__ out,
                                                        float *__restrict__ lse, int seq, int mbsz, int n, int nk, int d,
                                                        int causal, float scale) {
  const int lane = threadIdx.x & 63;
  size_t w = blockIdx.x * (size_t)4 + (threadIdx.x >> 6);
  if (w >= (size_t)mbsz * n * seq) return;
  const int i = w % seq, head = (w / seq) % n, b = w / ((size_t)seq * n);
  const int a = n * d, ak = nk * d;
  const size_t ld = (size_t)a + 2 * ak;
  const T *base = qkv + (size_t)b * seq * ld;
  const bool h0 = lane < d, h1 = lane + 64 < d;
  const T *qp = base + (size_t)i * ld + head * d;
  float q0 = h0 ? to_f32(qp[lane]) : 0.f, q1 = h1 ? to_f32(qp[lane + 64]) : 0.f;
  const int jend = causal ? i + 1 : seq;
  float m = -INFINITY, l = 0.f, o0 = 0.f, o1 = 0.f;
  for (int j = 0; j < jend; j++) {
    const T *kp = base + (size_t)j * ld + a + (head / (n / nk)) * d;
    const T *vp = kp + ak;
    float part = (h0 ? q0 * to_f32(kp[lane]) : 0.f) + (h1 ? q1 * to_f32(kp[lane + 64]) : 0.f);
    float sc = wave_sum(part) * scale;
    float mn = fmaxf(m, sc);
    float corr = expf(m - mn), p = expf(sc - mn);
    l = l * corr + p;
    o0 = o0 * corr + (h0 ? p * to_f32(vp[lane]) : 0.f);
    o1 = o1 * corr + (h1 ? p * to_f32(vp[lane + 64]) : 0.f);
    m = mn;
  }
  T *op = out + ((size_t)b * seq + i) * a + head * d;
  if (h0) op[lane] = from_f32<T>(o0 / l);
  if (h1) op[lane + 64] = from_f32<T>(o1 / l);
  if (lane == 0) lse[((size_t)b * n + head) * seq + i] = m + logf(l);
}

// dQ: wave per query row
template <typename T>
__global__ __launch_bounds__(256) void attn_bwd_dq_generic(const T *__restrict__ qkv, const float *__restrict__ lse,
                                                           const T *__restrict__ dout, const float *__restrict__ delta,
                                                           T *__restrict__ dqkv, int seq, int mbsz, int n, int nk, int d,
                                                           int causal, float scale) {
  const int lane = threadIdx.x & 63;
  size_t w = blockIdx.x * (size_t)4 + (threadIdx.x >> 6);
  if (w >= (size_t)mbsz * n * seq) return;
  const int i = w % seq, head = (w / seq) % n, b = w / ((size_t)seq * n);
  const int a = n * d, ak = nk * d;
  const size_t ld = (size_t)a + 2 * ak;
  const T *base = qkv + (size_t)b * seq * ld;
  const bool h0 = lane < d, h1 = lane + 64 < d;
  const T *qp = base + (size_t)i * ld + head * d;
  const T *dop = dout + ((size_t)b * seq + i) * a + head * d;
  float q0 = h0 ? to_f32(qp[lane]) : 0.f, q1 = h1 ? to_f32(qp[lane + 64]) : 0.f;
  float g0 = h0 ? to_f32(dop[lane]) : 0.f, g1 = h1 ? to_f32(dop[lane + 64]) : 0.f;
  const float L = lse[((size_t)b * n + head) * seq + i], D = delta[((size_t)b * n + head) * seq + i];
  const int jend = causal ? i + 1 : seq;
  float dq0 = 0.f, dq1 = 0.f;
  for (int j = 0; j < jend; j++) {
    const T *kp = base + (size_t)j * ld + a + (head / (n / nk)) * d;
    const T *vp = kp + ak;
    float k0 = h0 ? to_f32(kp[lane]) : 0.f, k1 = h1 ? to_f32(kp[lane + 64]) : 0.f;
    float v0 = h0 ? to_f32(vp[lane]) : 0.f, v1 = h1 ? to_f32(vp[lane + 64]) : 0.f;
    float sc = wave_sum(q0 * k0 + q1 * k1) * scale;
    float dp = wave_sum(g0 * v0 + g1 * v1);
    float ds = expf(sc - L) * (dp - D) * scale;
    dq0 += ds * k0;
    dq1 += ds * k1;
  }
  T *dqp = dqkv + ((size_t)b * seq + i) * ld + head * d;
  if (h0) dqp[lane] = from_f32<T>(dq0);
  if (h1) dqp[lane + 64] = from_f32<T>(dq1);
}

// dK, dV: wave per key row of a key / value head; sums over the query heads of its group in a fixed order
template <typename T>
__global__ __launch_bounds__(256) void attn_bwd_dkv_generic(const T *__restrict__ qkv, const float *__restrict__ lse,
                                                            const T *__restrict__ dout, const float *__restrict__ delta,
                                                            T *__restrict__ dqkv, int seq, int mbsz, int n, int nk, int d,
                                                            int causal, float scale) {
  const int lane = threadIdx.x & 63;
  size_t w = blockIdx.x * (size_t)4 + (threadIdx.x >> 6);
  if (w >= (size_t)mbsz * nk * seq) return;
  const int j = w % seq, kh = (w / seq) % nk, b = w / ((size_t)seq * nk);
  const int a = n * d, ak = nk * d, group = n / nk;
  const size_t ld = (size_t)a + 2 * ak;
  const T *base = qkv + (size_t)b * seq * ld;
  const bool h0 = lane < d, h1 = lane + 64 < d;
  const T *kp = base + (size_t)j * ld + a + kh * d;
  const T *vp = kp + ak;
  float k0 = h0 ? to_f32(kp[lane]) : 0.f, k1 = h1 ? to_f32(kp[lane + 64]) : 0.f;
  float v0 = h0 ? to_f32(vp[lane]) : 0.f, v1 = h1 ? to_f32(vp[lane + 64]) : 0.f;
  float dk0 = 0.f, dk1 = 0.f, dv0 = 0.f, dv1 = 0.f;
  for (int g = 0; g < group; g++) {
    const int head = kh * group + g;
    const float *Lr = lse + ((size_t)b * n + head) * seq, *Dr = delta + ((size_t)b * n + head) * seq;
    for (int i = causal ? j : 0; i < seq; i++) {
      const T *qp = base + (size_t)i * ld + head * d;
      const T *dop = dout + ((size_t)b * seq + i) * a + head * d;
      float q0 = h0 ? to_f32(qp[lane]) : 0.f, q1 = h1 ? to_f32(qp[lane + 64]) : 0.f;
      float g0 = h0 ? to_f32(dop[lane]) : 0.f, g1 = h1 ? to_f32(dop[lane + 64]) : 0.f;
      float sc = wave_sum(q0 * k0 + q1 * k1) * scale;
      float dp = wave_sum(g0 * v0 + g1 * v1);
      float p = expf(sc - Lr[i]);
      float ds = p * (dp - Dr[i]) * scale;
      dv0 += p * g0; dv1 += p * g1;
      dk0 += ds * q0; dk1 += ds * q1;
    }
  }
  T *dkp = dqkv + ((size_t)b * seq + j) * ld + a + kh * d;
  T *dvp = dkp + ak;
  if (h0) { dkp[lane] = from_f32<T>(dk0); dvp[lane] = from_f32<T>(dv0); }
  if (h1) { dkp[lane + 64] = from_f32<T>(dk1); dvp[lane + 64] = from_f32<T>(dv1); }
}

}  // namespace

int stp_launch_attn_fwd_generic(stp_ctx *ctx, const stp_layer_desc *d, const void *qkv, void *out, float *lse, hipStream_t s) {
  size_t waves = (size_t)d->mbsz * d->heads_local * d->seq;
  dim3 grid((waves + 3) / 4), block(256);
  float scale = 1.0f / sqrtf((float)d->head_dim);
  if (d->dtype == STP_BF16)
    hipLaunchKernelGGL(attn_fwd_generic<bf16_t>, grid, block, 0, s, (const bf16_t *)qkv, (bf16_t *)out, lse, d->seq, d->mbsz,
                       d->heads_local, stp_kv_heads(d), d->head_dim, d->causal, scale);
  else
    hipLaunchKernelGGL(attn_fwd_generic<float>, grid, block, 0, s, (const float *)qkv, (float *)out, lse, d->seq, d->mbsz,
                       d->heads_local, stp_kv_heads(d), d->head_dim, d->causal, scale);
  STP_LAUNCH_CHECK(ctx);
  return STP_OK;
}

int stp_launch_attn_bwd_generic(stp_ctx *ctx, const stp_layer_desc *d, const void *qkv, const void *out, const float *lse,
                                const void *dout, float *delta, void *dqkv, hipStream_t s) {
  int rc = stp_launch_rowdot(ctx, d, dout, out, delta, s);
  if (rc != STP_OK) return rc;
  size_t waves = (size_t)d->mbsz * d->heads_local * d->seq;
  dim3 grid((waves + 3) / 4), block(256);
  float scale = 1.0f / sqrtf((float)d->head_dim);
  const size_t waves_kv = (size_t)d->mbsz * stp_kv_heads(d) * d->seq;
  dim3 grid_kv((waves_kv + 3) / 4);
  if (d->dtype == STP_BF16) {
    hipLaunchKernelGGL(attn_bwd_dq_generic<bf16_t>, grid, block, 0, s, (const bf16_t *)qkv, lse, (const bf16_t *)dout, delta,
                       (bf16_t *)dqkv, d->seq, d->mbsz, d->heads_local, stp_kv_heads(d), d->head_dim, d->causal, scale);
    hipLaunchKernelGGL(attn_bwd_dkv_generic<bf16_t>, grid_kv, block, 0, s, (const bf16_t *)qkv, lse, (const bf16_t *)dout, delta,
                       (bf16_t *)dqkv, d->seq, d->mbsz, d->heads_local, stp_kv_heads(d), d->head_dim, d->causal, scale);
  } else {
    hipLaunchKernelGGL(attn_bwd_dq_generic<float>, grid, block, 0, s, (const float *)qkv, lse, (const float *)dout, delta,
                       (float *)dqkv, d->seq, d->mbsz, d->heads_local, stp_kv_heads(d), d->head_dim, d->causal, scale);
    hipLaunchKernelGGL(attn_bwd_dkv_generic<float>, grid_kv, block, 0, s, (const float *)qkv, lse, (const float *)dout, delta,
                       (float *)dqkv, d->seq, d->mbsz, d->heads_local, stp_kv_heads(d), d->head_dim, d->causal, scale);
  }
  STP_LAUNCH_CHECK(ctx);
  return STP_OK;
}

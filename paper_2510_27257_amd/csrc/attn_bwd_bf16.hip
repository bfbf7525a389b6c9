// Tiled attention backward for bf16 on the CDNA4 matrix cores (the attention part of the
// Attn unit's activation-gradient computation B; Section 3).
//
// Given Q, K, V, the forward's log-sum-exp L and delta = rowsum(dO o O):
//     P = exp(S - L),  S = Q K^T / sqrt(d)  (causal: key > query masked)
//     dV = P^T dO,  dP = dO V^T,  dS = P o (dP - delta),  dQ = dS K / sqrt(d),  dK = dS^T Q / sqrt(d)
// Two kernels, both deterministic (no atomics, no split accumulation):
//   * dkv: a workgroup owns 128 keys (32 per wave) and walks the query blocks; it forms S and dP
//     with the keys as MFMA columns, so the accumulator layout of P / dS is already the B-operand
//     layout of the two products dV^T += dO^T P and dK^T += Q^T dS.  dO^T / Q^T fragments come from
//     the [q][d] tiles through the transposing LDS read.
//   * dq: a workgroup owns 128 queries and walks the key blocks with the transposed tiles
//     S^T = K Q^T, dP^T = V dO^T (queries as MFMA columns: L and delta are per-lane scalars) and
//     dQ^T += K^T dS^T.
// S and dP are therefore formed twice (7 matrix products executed for the 4+1 the method needs);
// the price buys bit-reproducible gradients, which the braided == serialized check relies on.
// Tiles that are read both ways sit in LDS twice, once per pitch (144/272-byte rows for 16-byte
// fragment reads, +64-byte rows for transposing reads), so that both patterns are conflict free.
#include "common.h"

int stp_launch_rowdot(stp_ctx *ctx, const stp_layer_desc *d, const void *a, const void *b, float *delta, hipStream_t s);

namespace {

typedef s16x4_t __attribute__((address_space(3))) * lds_s16x4_ptr;
constexpr float LOG2E = 1.4426950408889634f;

template <int D> struct BG {
  static constexpr int kc = D + 8;    // pitch for 16-byte fragment reads
  static constexpr int tr = D + 32;   // pitch for transposing reads
  static constexpr int nld = 64 * D / 8 / 256;   // 16-byte chunks per thread for a 64 x D tile
};

// A-operand fragment (32 rows x 16 k) from a [row][k] tile, k contiguous
template <int P>
__device__ __forceinline__ bf16x8_t frag_kc(const bf16_t *tile, int row0, int k0, int lane) {
  return *reinterpret_cast<const bf16x8_t *>(tile + (row0 + (lane & 31)) * P + k0 + 8 * (lane >> 5));
}
// A-operand fragment whose 32 rows are the tile's COLUMNS c0.. and whose k-slots are tile rows
// r_lo + 4*(lane/32) + {0..3} and r_lo + 8 + 4*(lane/32) + {0..3}: the order in which a 32x32
// accumulator hands its rows to the next MFMA as a B operand.
template <int P>
__device__ __forceinline__ bf16x8_t frag_tr(const bf16_t *tile, int c0, int r_lo, int lane) {
  const bf16_t *p = tile + (r_lo + 4 * (lane >> 5) + ((lane & 15) >> 2)) * P + c0 + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
  s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p));
  s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p + 8 * P));
  s16x8_t v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8_t, v);
}

template <int D>
__device__ __forceinline__ void tile64_load(uint4 (&r)[BG<D>::nld], const bf16_t *__restrict__ base, size_t ld, int row0,
                                            int seq, int tid) {
#pragma unroll
  for (int i = 0; i < BG<D>::nld; i++) {
    int q = tid + 256 * i;
    int rr = q / (D / 8), c = (q % (D / 8)) * 8;
    int row = min(row0 + rr, seq - 1);                    // clamped: rows past the end are zeroed at store time
    r[i] = *reinterpret_cast<const uint4 *>(base + (size_t)row * ld + c);
  }
}
template <int D, int P>
__device__ __forceinline__ void tile64_store(const uint4 (&r)[BG<D>::nld], bf16_t *tile, int row0, int seq, int tid) {
#pragma unroll
  for (int i = 0; i < BG<D>::nld; i++) {
    int q = tid + 256 * i;
    int rr = q / (D / 8), c = (q % (D / 8)) * 8;
    const bool ok = row0 + rr < seq;
    uint4 v;
    v.x = ok ? r[i].x : 0u; v.y = ok ? r[i].y : 0u; v.z = ok ? r[i].z : 0u; v.w = ok ? r[i].w : 0u;
    *reinterpret_cast<uint4 *>(tile + rr * P + c) = v;
  }
}

// ---------------------------------------------------------------------------------------------
// dK, dV
// ---------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void attn_bwd_dkv_kernel(const bf16_t *__restrict__ qkv, const bf16_t *__restrict__ dout,
                                                           const float *__restrict__ lse, const float *__restrict__ delta,
                                                           bf16_t *__restrict__ dqkv, int seq, int n, int causal,
                                                           float scale) {
  using G = BG<D>;
  extern __shared__ __attribute__((aligned(16))) char smem_raw[];
  bf16_t *const q_kc = reinterpret_cast<bf16_t *>(smem_raw);
  bf16_t *const q_tr = q_kc + 64 * G::kc;
  bf16_t *const o_kc = q_tr + 64 * G::tr;
  bf16_t *const o_tr = o_kc + 64 * G::kc;
  float *const s_lse = reinterpret_cast<float *>(o_tr + 64 * G::tr);   // [64] log2-domain L
  float *const s_del = s_lse + 64;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lr = lane & 31, lg = lane >> 5;
  const int kvb = blockIdx.x, head = blockIdx.y, b = blockIdx.z;   // key block 0 has the longest walk and starts first
  const int a = n * D;
  const size_t ld = 3 * (size_t)a;
  const bf16_t *qbase = qkv + (size_t)b * seq * ld + head * D;
  const bf16_t *dobase = dout + (size_t)b * seq * a + head * D;
  const float *lse_b = lse + ((size_t)b * n + head) * seq;
  const float *del_b = delta + ((size_t)b * n + head) * seq;
  const int kv_wave0 = kvb * 128 + wave * 32;
  const int kvg = kv_wave0 + lr;
  const int kv_ld = min(kvg, seq - 1);
  const float scale_log2 = scale * LOG2E;

  // K and V rows of this lane as B-operand fragments (columns = keys)
  bf16x8_t kf[D / 16], vf[D / 16];
#pragma unroll
  for (int s = 0; s < D / 16; s++) {
    kf[s] = *reinterpret_cast<const bf16x8_t *>(qbase + a + (size_t)kv_ld * ld + 16 * s + 8 * lg);
    vf[s] = *reinterpret_cast<const bf16x8_t *>(qbase + 2 * a + (size_t)kv_ld * ld + 16 * s + 8 * lg);
  }
  f32x16_t dk[D / 32], dv[D / 32];
#pragma unroll
  for (int i = 0; i < D / 32; i++)
#pragma unroll
    for (int v = 0; v < 16; v++) { dk[i][v] = 0.f; dv[i][v] = 0.f; }

  const int q_start = causal ? (kvb * 128) / 64 : 0;       // first query block that can see these keys
  const int nqb = (seq + 63) / 64;
  uint4 rq[G::nld], ro[G::nld];
  float r_l = 0.f, r_d = 0.f;
  if (q_start < nqb) {
    tile64_load<D>(rq, qbase, ld, q_start * 64, seq, tid);
    tile64_load<D>(ro, dobase, a, q_start * 64, seq, tid);
    if (tid < 64) {
      int qi = q_start * 64 + tid;
      r_l = qi < seq ? lse_b[qi] * LOG2E : INFINITY;       // +inf makes P = 0 for rows past the end
      r_d = qi < seq ? del_b[qi] : 0.f;
    }
  }
  for (int qb = q_start; qb < nqb; qb++) {
    const int q0 = qb * 64;
    tile64_store<D, G::kc>(rq, q_kc, q0, seq, tid);
    tile64_store<D, G::tr>(rq, q_tr, q0, seq, tid);
    tile64_store<D, G::kc>(ro, o_kc, q0, seq, tid);
    tile64_store<D, G::tr>(ro, o_tr, q0, seq, tid);
    if (tid < 64) { s_lse[tid] = r_l; s_del[tid] = r_d; }
    __syncthreads();
    if (qb + 1 < nqb) {
      tile64_load<D>(rq, qbase, ld, q0 + 64, seq, tid);
      tile64_load<D>(ro, dobase, a, q0 + 64, seq, tid);
      if (tid < 64) {
        int qi = q0 + 64 + tid;
        r_l = qi < seq ? lse_b[qi] * LOG2E : INFINITY;
        r_d = qi < seq ? del_b[qi] : 0.f;
      }
    }
    const bool active = !causal || q0 + 63 >= kv_wave0;     // some query of the block sees some key of the wave
    if (active) {
      const bool need_mask = causal && q0 < kv_wave0 + 31;
#pragma unroll
      for (int qs = 0; qs < 2; qs++) {                     // two 32-query sub-blocks
        f32x16_t sacc, pacc;
#pragma unroll
        for (int v = 0; v < 16; v++) { sacc[v] = 0.f; pacc[v] = 0.f; }
#pragma unroll
        for (int s = 0; s < D / 16; s++) {
          sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_kc<G::kc>(q_kc, 32 * qs, 16 * s, lane), kf[s], sacc, 0, 0, 0);
          pacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_kc<G::kc>(o_kc, 32 * qs, 16 * s, lane), vf[s], pacc, 0, 0, 0);
        }
        // accumulator v of lane l: query q0 + 32*qs + 8*(v/4) + 4*(l/32) + v%4, key kv_wave0 + l%32
        bf16x8_t pf[2], sf[2];
#pragma unroll
        for (int j = 0; j < 4; j++) {
          const f32x4_t L4 = *reinterpret_cast<const f32x4_t *>(s_lse + 32 * qs + 8 * j + 4 * lg);
          const f32x4_t D4 = *reinterpret_cast<const f32x4_t *>(s_del + 32 * qs + 8 * j + 4 * lg);
#pragma unroll
          for (int r = 0; r < 4; r++) {
            const int v = 4 * j + r;
            float p = __builtin_amdgcn_exp2f(sacc[v] * scale_log2 - L4[r]);
            if (need_mask) {
              const int qi = q0 + 32 * qs + 8 * j + 4 * lg + r;
              if (qi < kvg) p = 0.f;
            }
            const float ds = p * (pacc[v] - D4[r]);
            pf[j >> 1][4 * (j & 1) + r] = (bf16_t)p;
            sf[j >> 1][4 * (j & 1) + r] = (bf16_t)ds;
          }
        }
        // dV^T[d, kv] += dO^T P ; dK^T[d, kv] += Q^T dS   (k = the 32 queries of the sub-block, two 16-steps)
#pragma unroll
        for (int t = 0; t < 2; t++)
#pragma unroll
          for (int db = 0; db < D / 32; db++) {
            dv[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_tr<G::tr>(o_tr, 32 * db, 32 * qs + 16 * t, lane), pf[t], dv[db], 0, 0, 0);
            dk[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_tr<G::tr>(q_tr, 32 * db, 32 * qs + 16 * t, lane), sf[t], dk[db], 0, 0, 0);
          }
      }
    }
    __syncthreads();
  }
  if (kvg < seq) {
    bf16_t *dkp = dqkv + ((size_t)b * seq + kvg) * ld + a + head * D;
    bf16_t *dvp = dkp + a;
#pragma unroll
    for (int db = 0; db < D / 32; db++)
#pragma unroll
      for (int j = 0; j < 4; j++) {
        bf16x4_t wk, wv;
#pragma unroll
        for (int r = 0; r < 4; r++) { wk[r] = (bf16_t)(dk[db][4 * j + r] * scale); wv[r] = (bf16_t)dv[db][4 * j + r]; }
        *reinterpret_cast<bf16x4_t *>(dkp + 32 * db + 8 * j + 4 * lg) = wk;
        *reinterpret_cast<bf16x4_t *>(dvp + 32 * db + 8 * j + 4 * lg) = wv;
      }
  }
}

// ---------------------------------------------------------------------------------------------
// dQ
// ---------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256, 2) void attn_bwd_dq_kernel(const bf16_t *__restrict__ qkv, const bf16_t *__restrict__ dout,
                                                             const float *__restrict__ lse, const float *__restrict__ delta,
                                                             bf16_t *__restrict__ dqkv, int seq, int n, int causal,
                                                             float scale) {
  using G = BG<D>;
  extern __shared__ __attribute__((aligned(16))) char smem_raw[];
  bf16_t *const k_kc = reinterpret_cast<bf16_t *>(smem_raw);
  bf16_t *const k_tr = k_kc + 64 * G::kc;
  bf16_t *const v_kc = k_tr + 64 * G::tr;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lr = lane & 31, lg = lane >> 5;
  const int nqblk = (seq + 127) / 128;
  const int qb = nqblk - 1 - blockIdx.x;                   // late query blocks walk the most keys: start them first
  const int head = blockIdx.y, b = blockIdx.z;
  const int a = n * D;
  const size_t ld = 3 * (size_t)a;
  const bf16_t *qbase = qkv + (size_t)b * seq * ld + head * D;
  const bf16_t *dobase = dout + (size_t)b * seq * a + head * D;
  const int q_wave0 = qb * 128 + wave * 32;
  const int qg = q_wave0 + lr;
  const int q_ld = min(qg, seq - 1);
  const float scale_log2 = scale * LOG2E;
  const float L2 = lse[((size_t)b * n + head) * seq + q_ld] * LOG2E;
  const float Dl = delta[((size_t)b * n + head) * seq + q_ld];

  bf16x8_t qf[D / 16], of[D / 16];
#pragma unroll
  for (int s = 0; s < D / 16; s++) {
    qf[s] = *reinterpret_cast<const bf16x8_t *>(qbase + (size_t)q_ld * ld + 16 * s + 8 * lg);
    of[s] = *reinterpret_cast<const bf16x8_t *>(dobase + (size_t)q_ld * a + 16 * s + 8 * lg);
  }
  f32x16_t dq[D / 32];
#pragma unroll
  for (int i = 0; i < D / 32; i++)
#pragma unroll
    for (int v = 0; v < 16; v++) dq[i][v] = 0.f;

  const int q_blk_end = min(seq, qb * 128 + 128);
  const int kv_end = causal ? q_blk_end : seq;
  const int nkb = (kv_end + 63) / 64;
  uint4 rk[G::nld], rv[G::nld];
  tile64_load<D>(rk, qbase + a, ld, 0, seq, tid);
  tile64_load<D>(rv, qbase + 2 * a, ld, 0, seq, tid);
  for (int kb = 0; kb < nkb; kb++) {
    const int kv0 = kb * 64;
    tile64_store<D, G::kc>(rk, k_kc, kv0, seq, tid);
    tile64_store<D, G::tr>(rk, k_tr, kv0, seq, tid);
    tile64_store<D, G::kc>(rv, v_kc, kv0, seq, tid);
    __syncthreads();
    if (kb + 1 < nkb) {
      tile64_load<D>(rk, qbase + a, ld, kv0 + 64, seq, tid);
      tile64_load<D>(rv, qbase + 2 * a, ld, kv0 + 64, seq, tid);
    }
    const bool active = !causal || kv0 <= q_wave0 + 31;
    if (active) {
      const bool need_mask = (causal && kv0 + 63 > q_wave0) || (kv0 + 64 > seq);
#pragma unroll
      for (int ks = 0; ks < 2; ks++) {                     // two 32-key sub-blocks
        f32x16_t sacc, pacc;
#pragma unroll
        for (int v = 0; v < 16; v++) { sacc[v] = 0.f; pacc[v] = 0.f; }
#pragma unroll
        for (int s = 0; s < D / 16; s++) {
          sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_kc<G::kc>(k_kc, 32 * ks, 16 * s, lane), qf[s], sacc, 0, 0, 0);
          pacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_kc<G::kc>(v_kc, 32 * ks, 16 * s, lane), of[s], pacc, 0, 0, 0);
        }
        // accumulator v of lane l: key kv0 + 32*ks + 8*(v/4) + 4*(l/32) + v%4, query q_wave0 + l%32
        bf16x8_t sf[2];
#pragma unroll
        for (int v = 0; v < 16; v++) {
          float p = __builtin_amdgcn_exp2f(sacc[v] * scale_log2 - L2);
          if (need_mask) {
            const int kv = kv0 + 32 * ks + 8 * (v >> 2) + 4 * lg + (v & 3);
            if ((causal && kv > qg) || kv >= seq) p = 0.f;
          }
          sf[v >> 3][v & 7] = (bf16_t)(p * (pacc[v] - Dl));
        }
#pragma unroll
        for (int t = 0; t < 2; t++)
#pragma unroll
          for (int db = 0; db < D / 32; db++)
            dq[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_tr<G::tr>(k_tr, 32 * db, 32 * ks + 16 * t, lane), sf[t], dq[db], 0, 0, 0);
      }
    }
    __syncthreads();
  }
  if (qg < seq) {
    bf16_t *dqp = dqkv + ((size_t)b * seq + qg) * ld + head * D;
#pragma unroll
    for (int db = 0; db < D / 32; db++)
#pragma unroll
      for (int j = 0; j < 4; j++) {
        bf16x4_t w;
#pragma unroll
        for (int r = 0; r < 4; r++) w[r] = (bf16_t)(dq[db][4 * j + r] * scale);
        *reinterpret_cast<bf16x4_t *>(dqp + 32 * db + 8 * j + 4 * lg) = w;
      }
  }
}

template <int D>
int launch_bwd(stp_ctx *ctx, const stp_layer_desc *d, const void *qkv, const float *lse, const void *dout, const float *delta,
               void *dqkv, hipStream_t s) {
  using G = BG<D>;
  constexpr size_t smem_kv = (size_t)2 * 64 * (G::kc + G::tr) * sizeof(bf16_t) + 128 * sizeof(float);
  constexpr size_t smem_q = (size_t)64 * (2 * G::kc + G::tr) * sizeof(bf16_t);
  auto kkv = attn_bwd_dkv_kernel<D>;
  auto kq = attn_bwd_dq_kernel<D>;
  static bool attr_set = false;
  if (!attr_set) {
    STP_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(kkv), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem_kv));
    STP_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(kq), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem_q));
    attr_set = true;
  }
  const float scale = 1.0f / sqrtf((float)D);
  dim3 grid((d->seq + 127) / 128, d->heads_local, d->mbsz), block(256);
  hipLaunchKernelGGL(kkv, grid, block, smem_kv, s, (const bf16_t *)qkv, (const bf16_t *)dout, lse, delta, (bf16_t *)dqkv, d->seq,
                     d->heads_local, d->causal, scale);
  STP_LAUNCH_CHECK(ctx);
  hipLaunchKernelGGL(kq, grid, block, smem_q, s, (const bf16_t *)qkv, (const bf16_t *)dout, lse, delta, (bf16_t *)dqkv, d->seq,
                     d->heads_local, d->causal, scale);
  STP_LAUNCH_CHECK(ctx);
  return STP_OK;
}

}  // namespace

int stp_launch_attn_bwd_bf16(stp_ctx *ctx, const stp_layer_desc *d, const void *qkv, const void *out, const float *lse,
                             const void *dout, float *delta, void *dqkv, hipStream_t s) {
  int rc = stp_launch_rowdot(ctx, d, dout, out, delta, s);
  if (rc != STP_OK) return rc;
  if (d->head_dim == 128) return launch_bwd<128>(ctx, d, qkv, lse, dout, delta, dqkv, s);
  if (d->head_dim == 64) return launch_bwd<64>(ctx, d, qkv, lse, dout, delta, dqkv, s);
  return stp_fail(ctx, STP_ESHAPE, "bf16 attention needs head_dim 64 or 128%s");
}

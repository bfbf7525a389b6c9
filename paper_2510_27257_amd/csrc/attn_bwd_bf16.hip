// Tiled attention backward for bf16 on the CDNA4 matrix cores (the attention part of the
// Attn unit's activation-gradient computation B; Section 3).
//
// Given Q, K, V, the forward's log-sum-exp L and delta = rowsum(dO o O):
//     P = exp(S - L),  S = Q K^T / sqrt(d)  (causal: key > query masked)
//     dV = P^T dO,  dP = dO V^T,  dS = P o (dP - delta),  dQ = dS K / sqrt(d),  dK = dS^T Q / sqrt(d)
// Two kernels, both deterministic (no atomics):
//   * dkv: a workgroup owns 128 keys and one CHUNK of up to 1024 queries; 8 waves = 4 key sub-tiles
//     (32 keys) x 2 halves of each 64-query step.  S and dP are formed with the keys as MFMA columns,
//     so the accumulator layout of P / dS is already the B-operand layout of dV^T += dO^T P and
//     dK^T += Q^T dS.  dO^T / Q^T fragments come from the [q][d] tiles through the transposing LDS read.
//   * dq: a workgroup owns 128 queries and one chunk of up to 1024 keys; 8 waves = 4 query sub-tiles
//     x 2 halves of each 128-key step, with the transposed tiles S^T = K Q^T, dP^T = V dO^T (queries
//     as MFMA columns: L and delta are per-lane scalars) and dQ^T += K^T dS^T.
// In both, the two wave halves are summed through LDS, every chunk writes an fp32 partial, and a
// small combine kernel adds the chunks in a fixed order.  Chunking balances the causal triangle over
// the 256 compute units; the 8-wave layout puts two waves on every SIMD so one wave's exponentials
// overlap the other's MFMAs.  S and dP are formed twice (7 matrix products executed for the 5 the
// method needs): the price of bit-reproducible gradients without atomics.
// Tiles that are read both ways sit in LDS twice, once per pitch (16-byte fragment reads want a
// +16-byte row pitch, transposing reads a +64-byte one), so both patterns are bank-conflict free.
#include "common.h"

int stp_launch_rowdot(stp_ctx *ctx, const stp_layer_desc *d, const void *a, const void *b, float *delta, hipStream_t s);

namespace {

typedef s16x4_t __attribute__((address_space(3))) * lds_s16x4_ptr;
constexpr float LOG2E = 1.4426950408889634f;
constexpr int KVB = 128;    // keys per dkv workgroup / per dq step
constexpr int QSTEP = 64;   // queries per dkv step
constexpr int CHQ = 16;     // dkv: steps per chunk (1024 queries)
constexpr int CHK = 8;      // dq: 128-key steps per chunk (1024 keys)

template <int D> struct BG {
  static constexpr int kc = D + 8;    // pitch for 16-byte fragment reads
  static constexpr int tr = D + 32;   // pitch for transposing reads
};

// fragment (32 rows x 16 k) from a [row][k] tile, k contiguous: lane supplies row row0 + l%32, k0 + 8*(l/32)..+7
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

// ROWS x D tile, 512 threads: registers <- global (rows clamped to seq-1), LDS <- registers (rows past seq zeroed)
template <int ROWS, int D, int NLD>
__device__ __forceinline__ void tile_load(uint4 (&r)[NLD], const bf16_t *__restrict__ base, size_t ld, int row0, int seq, int tid) {
  static_assert(NLD == ROWS * D / 8 / 512, "register count");
#pragma unroll
  for (int i = 0; i < NLD; i++) {
    int q = tid + 512 * i;
    int rr = q / (D / 8), c = (q % (D / 8)) * 8;
    int row = min(row0 + rr, seq - 1);
    r[i] = *reinterpret_cast<const uint4 *>(base + (size_t)row * ld + c);
  }
}
template <int D, int P, int NLD>
__device__ __forceinline__ void tile_store(const uint4 (&r)[NLD], bf16_t *tile, int row0, int seq, int tid) {
#pragma unroll
  for (int i = 0; i < NLD; i++) {
    int q = tid + 512 * i;
    int rr = q / (D / 8), c = (q % (D / 8)) * 8;
    const bool ok = row0 + rr < seq;
    uint4 v;
    v.x = ok ? r[i].x : 0u; v.y = ok ? r[i].y : 0u; v.z = ok ? r[i].z : 0u; v.w = ok ? r[i].w : 0u;
    *reinterpret_cast<uint4 *>(tile + rr * P + c) = v;
  }
}

__host__ __device__ inline int dkv_first_step(int kvb, int causal) { return causal ? (kvb * KVB) / QSTEP : 0; }
__host__ __device__ inline int dq_steps(int qb, int seq, int causal) {
  int kv_end = causal ? (seq < qb * 128 + 128 ? seq : qb * 128 + 128) : seq;
  return (kv_end + KVB - 1) / KVB;
}

// ---------------------------------------------------------------------------------------------
// dK, dV partials.  piece layout: dK [128][D] fp32, then dV [128][D] fp32
// ---------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(512) void attn_bwd_dkv_kernel(const bf16_t *__restrict__ qkv, const bf16_t *__restrict__ dout,
                                                           const float *__restrict__ lse, const float *__restrict__ delta,
                                                           float *__restrict__ part, int seq, int n, int causal,
                                                           int max_chunks, float scale) {
  using G = BG<D>;
  extern __shared__ __attribute__((aligned(16))) char smem_raw[];
  bf16_t *const k_kc = reinterpret_cast<bf16_t *>(smem_raw);
  bf16_t *const v_kc = k_kc + KVB * G::kc;
  bf16_t *const q_kc = v_kc + KVB * G::kc;
  bf16_t *const q_tr = q_kc + QSTEP * G::kc;
  bf16_t *const o_kc = q_tr + QSTEP * G::tr;
  bf16_t *const o_tr = o_kc + QSTEP * G::kc;
  float *const s_lse = reinterpret_cast<float *>(o_tr + QSTEP * G::tr);   // [64] log2-domain L
  float *const s_del = s_lse + QSTEP;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lr = lane & 31, lg = lane >> 5;
  const int ksub = wave & 3, qhalf = wave >> 2;
  const int kvb = blockIdx.x, chunk = blockIdx.y;      // key block 0 owns the most chunks and is scheduled first
  const int head = blockIdx.z % n, b = blockIdx.z / n;
  const int nq = (seq + QSTEP - 1) / QSTEP;
  const int s_begin = dkv_first_step(kvb, causal) + chunk * CHQ, s_end = min(nq, s_begin + CHQ);
  if (s_begin >= nq) return;

  const int a = n * D;
  const size_t ld = 3 * (size_t)a;
  const bf16_t *qbase = qkv + (size_t)b * seq * ld + head * D;
  const bf16_t *dobase = dout + (size_t)b * seq * a + head * D;
  const float *lse_b = lse + ((size_t)b * n + head) * seq;
  const float *del_b = delta + ((size_t)b * n + head) * seq;
  const int kv_wave0 = kvb * KVB + ksub * 32;
  const int kvg = kv_wave0 + lr;
  const float scale_log2 = scale * LOG2E;

  // K and V of the 128 keys: loaded once
  {
    uint4 rk[KVB * D / 8 / 512], rv[KVB * D / 8 / 512];
    tile_load<KVB, D>(rk, qbase + a, ld, kvb * KVB, seq, tid);
    tile_load<KVB, D>(rv, qbase + 2 * a, ld, kvb * KVB, seq, tid);
    tile_store<D, G::kc>(rk, k_kc, kvb * KVB, seq, tid);
    tile_store<D, G::kc>(rv, v_kc, kvb * KVB, seq, tid);
  }
  f32x16_t dk[D / 32], dv[D / 32];
#pragma unroll
  for (int i = 0; i < D / 32; i++)
#pragma unroll
    for (int v = 0; v < 16; v++) { dk[i][v] = 0.f; dv[i][v] = 0.f; }

  uint4 rq[QSTEP * D / 8 / 512], ro[QSTEP * D / 8 / 512];
  float r_l = 0.f, r_d = 0.f;
  tile_load<QSTEP, D>(rq, qbase, ld, s_begin * QSTEP, seq, tid);
  tile_load<QSTEP, D>(ro, dobase, a, s_begin * QSTEP, seq, tid);
  if (tid < QSTEP) {
    int qi = s_begin * QSTEP + tid;
    r_l = qi < seq ? lse_b[qi] * LOG2E : INFINITY;       // +inf makes P = 0 for rows past the end
    r_d = qi < seq ? del_b[qi] : 0.f;
  }
  for (int st = s_begin; st < s_end; st++) {
    const int q0 = st * QSTEP;
    tile_store<D, G::kc>(rq, q_kc, q0, seq, tid);
    tile_store<D, G::tr>(rq, q_tr, q0, seq, tid);
    tile_store<D, G::kc>(ro, o_kc, q0, seq, tid);
    tile_store<D, G::tr>(ro, o_tr, q0, seq, tid);
    if (tid < QSTEP) { s_lse[tid] = r_l; s_del[tid] = r_d; }
    __syncthreads();
    if (st + 1 < s_end) {
      tile_load<QSTEP, D>(rq, qbase, ld, q0 + QSTEP, seq, tid);
      tile_load<QSTEP, D>(ro, dobase, a, q0 + QSTEP, seq, tid);
      if (tid < QSTEP) {
        int qi = q0 + QSTEP + tid;
        r_l = qi < seq ? lse_b[qi] * LOG2E : INFINITY;
        r_d = qi < seq ? del_b[qi] : 0.f;
      }
    }
    const int qs0 = q0 + 32 * qhalf;                        // this wave's 32 queries of the step
    const bool active = !causal || qs0 + 31 >= kv_wave0;    // some query sees some key of the wave
    if (active) {
      const bool need_mask = causal && qs0 < kv_wave0 + 31;
      f32x16_t sacc, pacc;
#pragma unroll
      for (int v = 0; v < 16; v++) { sacc[v] = 0.f; pacc[v] = 0.f; }
#pragma unroll
      for (int s = 0; s < D / 16; s++) {
        sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_kc<G::kc>(q_kc, 32 * qhalf, 16 * s, lane),
                                                       frag_kc<G::kc>(k_kc, 32 * ksub, 16 * s, lane), sacc, 0, 0, 0);
        pacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_kc<G::kc>(o_kc, 32 * qhalf, 16 * s, lane),
                                                       frag_kc<G::kc>(v_kc, 32 * ksub, 16 * s, lane), pacc, 0, 0, 0);
      }
      // accumulator v of lane l: query qs0 + 8*(v/4) + 4*(l/32) + v%4, key kv_wave0 + l%32
      bf16x8_t pf[2], sf[2];
#pragma unroll
      for (int j = 0; j < 4; j++) {
        const f32x4_t L4 = *reinterpret_cast<const f32x4_t *>(s_lse + 32 * qhalf + 8 * j + 4 * lg);
        const f32x4_t D4 = *reinterpret_cast<const f32x4_t *>(s_del + 32 * qhalf + 8 * j + 4 * lg);
#pragma unroll
        for (int r = 0; r < 4; r++) {
          const int v = 4 * j + r;
          float p = __builtin_amdgcn_exp2f(sacc[v] * scale_log2 - L4[r]);
          if (need_mask) {
            const int qi = qs0 + 8 * j + 4 * lg + r;
            if (qi < kvg) p = 0.f;
          }
          const float ds = p * (pacc[v] - D4[r]);
          pf[j >> 1][4 * (j & 1) + r] = (bf16_t)p;
          sf[j >> 1][4 * (j & 1) + r] = (bf16_t)ds;
        }
      }
      // dV^T[d, kv] += dO^T P ; dK^T[d, kv] += Q^T dS   (k = the 32 queries, two 16-steps)
#pragma unroll
      for (int t = 0; t < 2; t++)
#pragma unroll
        for (int db = 0; db < D / 32; db++) {
          dv[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_tr<G::tr>(o_tr, 32 * db, 32 * qhalf + 16 * t, lane), pf[t], dv[db], 0, 0, 0);
          dk[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_tr<G::tr>(q_tr, 32 * db, 32 * qhalf + 16 * t, lane), sf[t], dk[db], 0, 0, 0);
        }
    }
    __syncthreads();
  }
  // ---- sum the two query halves through LDS (upper half -> lower half), write the chunk's partial
  float *red = reinterpret_cast<float *>(smem_raw);        // [4][D][64]: dk rows 0..D/2-1, dv rows D/2..D-1 per key sub-tile
  if (qhalf == 1) {
#pragma unroll
    for (int i = 0; i < D / 32; i++)
#pragma unroll
      for (int v = 0; v < 16; v++) {
        red[(ksub * D + i * 16 + v) * 64 + lane] = dk[i][v];
        red[(ksub * D + D / 2 + i * 16 + v) * 64 + lane] = dv[i][v];
      }
  }
  __syncthreads();
  if (qhalf == 0 && kvg < seq) {
    const int nkvb = (seq + KVB - 1) / KVB;
    const size_t piece = (((size_t)b * n + head) * nkvb + kvb) * max_chunks + chunk;
    float *pk = part + piece * (size_t)(2 * KVB * D) + (size_t)(ksub * 32 + lr) * D;
    float *pv = pk + (size_t)KVB * D;
#pragma unroll
    for (int i = 0; i < D / 32; i++)
#pragma unroll
      for (int j = 0; j < 4; j++) {
        f32x4_t wk, wv;
#pragma unroll
        for (int r = 0; r < 4; r++) {
          const int v = 4 * j + r;
          wk[r] = dk[i][v] + red[(ksub * D + i * 16 + v) * 64 + lane];
          wv[r] = dv[i][v] + red[(ksub * D + D / 2 + i * 16 + v) * 64 + lane];
        }
        *reinterpret_cast<f32x4_t *>(pk + 32 * i + 8 * j + 4 * lg) = wk;
        *reinterpret_cast<f32x4_t *>(pv + 32 * i + 8 * j + 4 * lg) = wv;
      }
  }
}

// dK = scale * sum_c, dV = sum_c over the chunks of a key block (fixed order).  One thread per 8 columns of a key row.
template <int D>
__global__ __launch_bounds__(256) void attn_bwd_dkv_combine_kernel(const float *__restrict__ part, bf16_t *__restrict__ dqkv,
                                                                   int seq, int n, int mbsz, int causal, int max_chunks,
                                                                   float scale) {
  const size_t idx = blockIdx.x * (size_t)256 + threadIdx.x;
  constexpr int CPR = D / 8;
  if (idx >= (size_t)mbsz * n * seq * CPR) return;
  const int c8 = (idx % CPR) * 8;
  const size_t row = idx / CPR;
  const int kv = row % seq, head = (row / seq) % n, b = row / ((size_t)seq * n);
  const int kvb = kv / KVB, kloc = kv % KVB;
  const int nkvb = (seq + KVB - 1) / KVB, nq = (seq + QSTEP - 1) / QSTEP;
  const int nch = (nq - dkv_first_step(kvb, causal) + CHQ - 1) / CHQ;
  const float *p0 = part + ((((size_t)b * n + head) * nkvb + kvb) * max_chunks) * (size_t)(2 * KVB * D) + (size_t)kloc * D + c8;
  float sk[8] = {0, 0, 0, 0, 0, 0, 0, 0}, sv[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  for (int c = 0; c < nch; c++) {
    float a8[8], b8[8];
    Vec8<float>::load(p0 + (size_t)c * (2 * KVB * D), a8);
    Vec8<float>::load(p0 + (size_t)c * (2 * KVB * D) + (size_t)KVB * D, b8);
#pragma unroll
    for (int e = 0; e < 8; e++) { sk[e] += a8[e]; sv[e] += b8[e]; }
  }
#pragma unroll
  for (int e = 0; e < 8; e++) sk[e] *= scale;
  const int a = n * D;
  bf16_t *dkp = dqkv + ((size_t)b * seq + kv) * (3 * (size_t)a) + a + head * D + c8;
  Vec8<bf16_t>::store(dkp, sk);
  Vec8<bf16_t>::store(dkp + a, sv);
}

// ---------------------------------------------------------------------------------------------
// dQ partials.  piece layout: dQ [128][D] fp32 (unscaled)
// ---------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(512) void attn_bwd_dq_kernel(const bf16_t *__restrict__ qkv, const bf16_t *__restrict__ dout,
                                                          const float *__restrict__ lse, const float *__restrict__ delta,
                                                          float *__restrict__ part, int seq, int n, int causal, int max_chunks,
                                                          float scale) {
  using G = BG<D>;
  extern __shared__ __attribute__((aligned(16))) char smem_raw[];
  bf16_t *const k_kc = reinterpret_cast<bf16_t *>(smem_raw);
  bf16_t *const k_tr = k_kc + KVB * G::kc;
  bf16_t *const v_kc = k_tr + KVB * G::tr;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lr = lane & 31, lg = lane >> 5;
  const int qsub = wave & 3, half = wave >> 2;
  const int nqblk = (seq + 127) / 128;
  const int qb = nqblk - 1 - blockIdx.x;                   // late query blocks own the most chunks: start them first
  const int chunk = blockIdx.y;
  const int head = blockIdx.z % n, b = blockIdx.z / n;
  const int nsteps = dq_steps(qb, seq, causal);
  const int s_begin = chunk * CHK, s_end = min(nsteps, s_begin + CHK);
  if (s_begin >= nsteps) return;

  const int a = n * D;
  const size_t ld = 3 * (size_t)a;
  const bf16_t *qbase = qkv + (size_t)b * seq * ld + head * D;
  const bf16_t *dobase = dout + (size_t)b * seq * a + head * D;
  const int q_wave0 = qb * 128 + qsub * 32;
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

  uint4 rk[KVB * D / 8 / 512], rv[KVB * D / 8 / 512];
  tile_load<KVB, D>(rk, qbase + a, ld, s_begin * KVB, seq, tid);
  tile_load<KVB, D>(rv, qbase + 2 * a, ld, s_begin * KVB, seq, tid);
  for (int st = s_begin; st < s_end; st++) {
    const int kvt = st * KVB;
    tile_store<D, G::kc>(rk, k_kc, kvt, seq, tid);
    tile_store<D, G::tr>(rk, k_tr, kvt, seq, tid);
    tile_store<D, G::kc>(rv, v_kc, kvt, seq, tid);
    __syncthreads();
    if (st + 1 < s_end) {
      tile_load<KVB, D>(rk, qbase + a, ld, kvt + KVB, seq, tid);
      tile_load<KVB, D>(rv, qbase + 2 * a, ld, kvt + KVB, seq, tid);
    }
    const int kv0 = kvt + 64 * half;                         // this wave's 64 keys of the step
    const bool active = kv0 < seq && (!causal || kv0 <= q_wave0 + 31);
    if (active) {
      const bool need_mask = (causal && kv0 + 63 > q_wave0) || (kv0 + 64 > seq);
#pragma unroll
      for (int ks = 0; ks < 2; ks++) {                     // two 32-key sub-blocks
        const int r0 = 64 * half + 32 * ks;                // first tile row of the sub-block
        f32x16_t sacc, pacc;
#pragma unroll
        for (int v = 0; v < 16; v++) { sacc[v] = 0.f; pacc[v] = 0.f; }
#pragma unroll
        for (int s = 0; s < D / 16; s++) {
          sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_kc<G::kc>(k_kc, r0, 16 * s, lane), qf[s], sacc, 0, 0, 0);
          pacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_kc<G::kc>(v_kc, r0, 16 * s, lane), of[s], pacc, 0, 0, 0);
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
            dq[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_tr<G::tr>(k_tr, 32 * db, r0 + 16 * t, lane), sf[t], dq[db], 0, 0, 0);
      }
    }
    __syncthreads();
  }
  float *red = reinterpret_cast<float *>(smem_raw);        // [4][D/2][64]
  if (half == 1) {
#pragma unroll
    for (int i = 0; i < D / 32; i++)
#pragma unroll
      for (int v = 0; v < 16; v++) red[(qsub * (D / 2) + i * 16 + v) * 64 + lane] = dq[i][v];
  }
  __syncthreads();
  if (half == 0 && qg < seq) {
    const size_t piece = (((size_t)b * n + head) * nqblk + qb) * max_chunks + chunk;
    float *pq = part + piece * (size_t)(128 * D) + (size_t)(qsub * 32 + lr) * D;
#pragma unroll
    for (int i = 0; i < D / 32; i++)
#pragma unroll
      for (int j = 0; j < 4; j++) {
        f32x4_t w;
#pragma unroll
        for (int r = 0; r < 4; r++) {
          const int v = 4 * j + r;
          w[r] = dq[i][v] + red[(qsub * (D / 2) + i * 16 + v) * 64 + lane];
        }
        *reinterpret_cast<f32x4_t *>(pq + 32 * i + 8 * j + 4 * lg) = w;
      }
  }
}

template <int D>
__global__ __launch_bounds__(256) void attn_bwd_dq_combine_kernel(const float *__restrict__ part, bf16_t *__restrict__ dqkv,
                                                                  int seq, int n, int mbsz, int causal, int max_chunks,
                                                                  float scale) {
  const size_t idx = blockIdx.x * (size_t)256 + threadIdx.x;
  constexpr int CPR = D / 8;
  if (idx >= (size_t)mbsz * n * seq * CPR) return;
  const int c8 = (idx % CPR) * 8;
  const size_t row = idx / CPR;
  const int q = row % seq, head = (row / seq) % n, b = row / ((size_t)seq * n);
  const int qb = q / 128, qloc = q % 128;
  const int nqblk = (seq + 127) / 128;
  const int nch = (dq_steps(qb, seq, causal) + CHK - 1) / CHK;
  const float *p0 = part + ((((size_t)b * n + head) * nqblk + qb) * max_chunks) * (size_t)(128 * D) + (size_t)qloc * D + c8;
  float sq[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  for (int c = 0; c < nch; c++) {
    float a8[8];
    Vec8<float>::load(p0 + (size_t)c * (128 * D), a8);
#pragma unroll
    for (int e = 0; e < 8; e++) sq[e] += a8[e];
  }
#pragma unroll
  for (int e = 0; e < 8; e++) sq[e] *= scale;
  const int a = n * D;
  Vec8<bf16_t>::store(dqkv + ((size_t)b * seq + q) * (3 * (size_t)a) + head * D + c8, sq);
}

inline int dkv_max_chunks(int seq) { return ((seq + QSTEP - 1) / QSTEP + CHQ - 1) / CHQ; }
inline int dq_max_chunks(int seq, int causal) { return (dq_steps((seq + 127) / 128 - 1, seq, causal) + CHK - 1) / CHK; }

template <int D>
int launch_bwd(stp_ctx *ctx, const stp_layer_desc *d, const void *qkv, const float *lse, const void *dout, const float *delta,
               void *dqkv, float *ws, size_t ws_bytes, hipStream_t s) {
  using G = BG<D>;
  constexpr size_t smem_kv = (size_t)(2 * KVB * G::kc + 2 * QSTEP * (G::kc + G::tr)) * sizeof(bf16_t) + 2 * QSTEP * sizeof(float);
  constexpr size_t smem_q = (size_t)KVB * (2 * G::kc + G::tr) * sizeof(bf16_t);
  static_assert(smem_kv <= 160 * 1024 && smem_kv >= (size_t)4 * D * 64 * sizeof(float), "dkv LDS budget");
  static_assert(smem_q <= 160 * 1024 && smem_q >= (size_t)4 * (D / 2) * 64 * sizeof(float), "dq LDS budget");
  auto kkv = attn_bwd_dkv_kernel<D>;
  auto kq = attn_bwd_dq_kernel<D>;
  static bool attr_set = false;
  if (!attr_set) {
    STP_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(kkv), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem_kv));
    STP_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(kq), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem_q));
    attr_set = true;
  }
  const float scale = 1.0f / sqrtf((float)D);
  const int nkvb = (d->seq + KVB - 1) / KVB, nqb = (d->seq + 127) / 128;
  const int mc_kv = dkv_max_chunks(d->seq), mc_q = dq_max_chunks(d->seq, d->causal);
  const size_t bh = (size_t)d->mbsz * d->heads_local;
  const size_t need_kv = bh * nkvb * mc_kv * 2 * KVB * D * sizeof(float), need_q = bh * nqb * mc_q * 128 * D * sizeof(float);
  const size_t need = need_kv > need_q ? need_kv : need_q;
  if (!ws || ws_bytes < need)
    return stp_fail(ctx, STP_ENOSPACE, "attention backward: workspace lane too small%s (need %ld bytes)", "", (long)need);
  const size_t rows8 = bh * d->seq * (D / 8);
  hipLaunchKernelGGL(kkv, dim3(nkvb, mc_kv, (unsigned)bh), dim3(512), smem_kv, s, (const bf16_t *)qkv, (const bf16_t *)dout, lse,
                     delta, ws, d->seq, d->heads_local, d->causal, mc_kv, scale);
  STP_LAUNCH_CHECK(ctx);
  hipLaunchKernelGGL(attn_bwd_dkv_combine_kernel<D>, dim3((rows8 + 255) / 256), dim3(256), 0, s, ws, (bf16_t *)dqkv, d->seq,
                     d->heads_local, d->mbsz, d->causal, mc_kv, scale);
  STP_LAUNCH_CHECK(ctx);
  hipLaunchKernelGGL(kq, dim3(nqb, mc_q, (unsigned)bh), dim3(512), smem_q, s, (const bf16_t *)qkv, (const bf16_t *)dout, lse, delta,
                     ws, d->seq, d->heads_local, d->causal, mc_q, scale);
  STP_LAUNCH_CHECK(ctx);
  hipLaunchKernelGGL(attn_bwd_dq_combine_kernel<D>, dim3((rows8 + 255) / 256), dim3(256), 0, s, ws, (bf16_t *)dqkv, d->seq,
                     d->heads_local, d->mbsz, d->causal, mc_q, scale);
  STP_LAUNCH_CHECK(ctx);
  return STP_OK;
}

}  // namespace

size_t stp_attn_bwd_ws_bytes(const stp_layer_desc *d) {
  const int nkvb = (d->seq + KVB - 1) / KVB, nqb = (d->seq + 127) / 128;
  const size_t bh = (size_t)d->mbsz * d->heads_local;
  const size_t need_kv = bh * nkvb * dkv_max_chunks(d->seq) * 2 * KVB * d->head_dim * sizeof(float);
  const size_t need_q = bh * nqb * dq_max_chunks(d->seq, d->causal) * 128 * d->head_dim * sizeof(float);
  return need_kv > need_q ? need_kv : need_q;
}

int stp_launch_attn_bwd_bf16(stp_ctx *ctx, const stp_layer_desc *d, const void *qkv, const void *out, const float *lse,
                             const void *dout, float *delta, void *dqkv, float *ws, size_t ws_bytes, hipStream_t s) {
  int rc = stp_launch_rowdot(ctx, d, dout, out, delta, s);
  if (rc != STP_OK) return rc;
  if (d->head_dim == 128) return launch_bwd<128>(ctx, d, qkv, lse, dout, delta, dqkv, ws, ws_bytes, s);
  if (d->head_dim == 64) return launch_bwd<64>(ctx, d, qkv, lse, dout, delta, dqkv, ws, ws_bytes, s);
  return stp_fail(ctx, STP_ESHAPE, "bf16 attention needs head_dim 64 or 128%s");
}

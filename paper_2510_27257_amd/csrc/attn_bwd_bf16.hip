// Tiled attention backward for bf16 on the CDNA4 matrix cores (the attention part of the
// Attn unit's activation-gradient computation B; Section 3).
//
// Given Q, K, V, the forward's log-sum-exp L and delta = rowsum(dO o O):
//     P = exp(S - L),  S = Q K^T / sqrt(d)  (causal: key > query masked)
//     dV = P^T dO,  dP = dO V^T,  dS = P o (dP - delta),  dQ = dS K / sqrt(d),  dK = dS^T Q / sqrt(d)
// Two kernel bodies, both deterministic (no atomics), run by one launch when the query and key / value head
// counts are equal (their workgroups then fill each other's idle compute units) and by two launches otherwise:
//   * dkv: a workgroup owns 128 keys and one CHUNK of steps of 64 queries; 8 waves = 4 key sub-tiles
//     (32 keys) x 2 halves of each 64-query step.  S and dP are formed with the keys as MFMA columns,
//     so the accumulator layout of P / dS is already the B-operand layout of dV^T += dO^T P and
//     dK^T += Q^T dS.  dO^T / Q^T fragments come from the [q][d] tiles through the transposing LDS read.
//   * dq: a workgroup owns 128 queries and one chunk of steps of 128 keys; 8 waves = 4 query sub-tiles
//     x 2 halves of each 128-key step, with the transposed tiles S^T = K Q^T, dP^T = V dO^T (queries
//     as MFMA columns: L and delta are per-lane scalars) and dQ^T += K^T dS^T.
// Grouped-query attention: a key / value head serves n / nk query heads.  dq only changes its tile addresses;
// a dkv workgroup runs over the (query head of the group, query step) pairs of its key block, so dK and dV
// collect the whole group in a fixed order.
// In both, the two wave halves are summed through LDS, every chunk writes an fp32 partial, and a
// small combine kernel adds the chunks in a fixed order.  Chunking balances the causal triangle over
// the 256 compute units (chunk length and dispatch order, longest first, come from the host-side plan); the 8-wave layout puts two waves on every SIMD so one wave's exponentials
// overlap the other's MFMAs.  S and dP are formed twice (7 matrix products executed for the 5 the
// method needs): the price of bit-reproducible gradients without atomics.
// Tiles go global -> LDS directly (buffer_load ... lds) and sit there once, unpadded ([row][D]); the
// 16-byte chunks of a row are permuted by an XOR, slot = chunk ^ swz(row), applied on the global side
// of the load and undone in the fragment addresses.  swz is chosen so that both access patterns are
// bank-conflict free: 16-byte fragment reads (16 consecutive rows, same chunk) and transposing
// ds_read_b64_tr_b16 reads (4 consecutive rows x 4 consecutive chunks).  Fragment reads are inline
// assembly with explicit waits, software-pipelined one MFMA group ahead.
#include "common.h"
#include "lds_dma.h"
#include <type_traits>
#include <vector>
#include <algorithm>

int stp_launch_rowdot(stp_ctx *ctx, const stp_layer_desc *d, const void *a, const void *b, float *delta, hipStream_t s);

namespace {

constexpr float LOG2E = 1.4426950408889634f;
constexpr int KVB = 128;    // keys per dkv workgroup / per dq step
constexpr int QSTEP = 64;   // queries per dkv step

template <int D> struct BG {
  static constexpr int RB = D * 2;        // bytes per tile row
  static constexpr int CPR = D / 8;       // 16-byte chunks per row
  static constexpr int RPI = 64 / CPR;    // rows covered by one direct-to-LDS wave instruction
  // chunk permutation of a tile row.  D = 128 (16 chunks, one row per 256 B): rows r..r+15 get 16 distinct
  // values and rows 4m..4m+3 differ in bits 2-3.  D = 64 (8 chunks, two rows per 256 B): the same for row pairs.
  static __device__ __forceinline__ int swz(int row) {
    if (D == 128) return ((row & 3) << 2) | ((row >> 2) & 3);
    const int x = row >> 1;
    return ((x & 1) << 2) | ((x >> 1) & 3);
  }
};

// Loads rows row0 .. row0+ROWS-1 (clamped to seq-1) of a [seq][ld] bf16 matrix, D columns from byte column col_bytes,
// into the swizzled LDS tile.  Every wave issues ROWS / RPI / 8 wave instructions.
template <int D, int ROWS>
__device__ __forceinline__ void dma_tile(__amdgpu_buffer_rsrc_t rs, char *tile, int row0, int seq, unsigned ld_bytes, unsigned col_bytes,
                                         int wave, int lane) {
  using G = BG<D>;
  constexpr int N = ROWS / G::RPI / 8;
  static_assert(N >= 1, "tile too small for 8 waves");
  // byte offset = min(uniform part + lane's row part, last row) + lane's column part: the lane parts do not
  // change from step to step, so a load costs an add, a min and an add; the LDS target is wave-uniform
  const int wave_s = __builtin_amdgcn_readfirstlane(wave);
  const unsigned uni = (unsigned)row0 * ld_bytes, last = (unsigned)(seq - 1) * ld_bytes;
#pragma unroll
  for (int j = 0; j < N; j++) {
    const int row = (wave * N + j) * G::RPI + lane / G::CPR, slot = lane % G::CPR;
    const unsigned row_part = (unsigned)row * ld_bytes, col_part = col_bytes + ((slot ^ G::swz(row)) * 16);
    dma_load16(rs, tile + (wave_s * N + j) * 1024, min(uni + row_part, last) + col_part, 0);
  }
}

// two 16-byte fragments (k-steps 2*SP and 2*SP+1) of tile rows ROW0 + lane%32; base = tile + lane part (see kc_lane)
template <int D, int ROW0, int SP>
__device__ __forceinline__ void read_kc2(u32x4_t &f0, u32x4_t &f1, unsigned base) {
  f0 = lds_read_b128<ROW0 * BG<D>::RB>(base ^ (32 * (2 * SP)));
  f1 = lds_read_b128<ROW0 * BG<D>::RB>(base ^ (32 * (2 * SP + 1)));
}
// lane part of a 16-byte fragment address: row lane%32 (+ a multiple of 32), k-step 0; XOR 32*s selects k-step s
template <int D>
__device__ __forceinline__ unsigned kc_lane(int lane) {
  const int lr = lane & 31, lg = lane >> 5;
  return lr * BG<D>::RB + ((lg ^ BG<D>::swz(lr)) * 16);
}
// Transposed fragment: A operand whose 32 rows are tile COLUMNS 32*db .. and whose k-slots are tile rows
// R0 + 4*(lane/32) + {0..3} and R0 + 8 + 4*(lane/32) + {0..3} (R0 a multiple of 16): the order in which a
// 32x32 accumulator hands its rows to the next MFMA as a B operand.  lo/hi = tile + lane parts (tr_lane).
template <int D, int R0>
__device__ __forceinline__ u32x4_t read_tr(unsigned lo, unsigned hi, int db) {
  u32x2_t a, b;
  const unsigned x = 64 * db;
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(a) : "v"(lo ^ x), "n"(R0 * BG<D>::RB));
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(b) : "v"(hi ^ x), "n"((R0 + 8) * BG<D>::RB));
  return __builtin_shufflevector(a, b, 0, 1, 2, 3);
}
template <int D>
__device__ __forceinline__ void tr_lane(int lane, unsigned &lo, unsigned &hi) {
  const int row = 4 * (lane >> 5) + ((lane & 15) >> 2);      // + R0 (multiple of 16: does not change swz)
  const int col = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);   // + 32 db (XOR 64*db on the address)
  lo = row * BG<D>::RB + (((col >> 3) ^ BG<D>::swz(row)) * 16) + (col & 7) * 2;
  hi = row * BG<D>::RB + (((col >> 3) ^ BG<D>::swz(row + 8)) * 16) + (col & 7) * 2;
}

__host__ __device__ inline int dkv_first_step(int kvb, int causal) { return causal ? (kvb * KVB) / QSTEP : 0; }
__host__ __device__ inline int dq_steps(int qb, int seq, int causal) {
  int kv_end = causal ? (seq < qb * 128 + 128 ? seq : qb * 128 + 128) : seq;
  return (kv_end + KVB - 1) / KVB;
}

#define STP_SB() __builtin_amdgcn_sched_barrier(0)

// ---------------------------------------------------------------------------------------------
// dK, dV partials.  piece layout: dK [128][D] fp32, then dV [128][D] fp32
// LDS: K [128][D], V [128][D] (resident), then a ring of two stages { Q [64][D], dO [64][D] }, then the
// ring of { lse [64], delta [64] } (fp32).
// ---------------------------------------------------------------------------------------------
template <int D>
__device__ __forceinline__ void dkv_body(const bf16_t *__restrict__ qkv, const bf16_t *__restrict__ dout,
                                         const float *__restrict__ lse, const float *__restrict__ delta,
                                         float *__restrict__ part, bf16_t *__restrict__ dqkv, int seq, int n, int nk, int causal,
                                         int max_chunks, int chunk_steps, float scale, int kvb, int chunk, int bz) {
  using G = BG<D>;
  constexpr int RB = G::RB;
  constexpr int KV_TILE = KVB * RB, Q_TILE = QSTEP * RB, STAGE = 2 * Q_TILE;
  constexpr int OFF_K = 0, OFF_V = KV_TILE, OFF_RING = 2 * KV_TILE, OFF_STAT = OFF_RING + 2 * STAGE;
  extern __shared__ __attribute__((aligned(1024))) char smem_raw[];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lr = lane & 31, lg = lane >> 5;
  const int ksub = wave & 3, qhalf = wave >> 2;
  const int kh = bz % nk, b = bz / nk;                     // key / value head
  const int group = n / nk;                                // query heads kh*group .. kh*group+group-1 share it
  const int nq = (seq + QSTEP - 1) / QSTEP;
  // the workgroup's steps run over (query head of the group, 64-query step): step u is query head
  // kh*group + u / nq_k, queries (first + u % nq_k) * 64 ..
  const int first = dkv_first_step(kvb, causal), nq_k = nq - first;
  const int s_begin = chunk * chunk_steps, s_end = min(group * nq_k, s_begin + chunk_steps);
  if (s_begin >= group * nq_k) return;
  const int ns = s_end - s_begin;

  const int a = n * D;
  const unsigned ldq = (unsigned)(n + 2 * nk) * D * 2u, ldo = (unsigned)a * 2u;       // row pitches in bytes
  const bf16_t *qkv_b = qkv + (size_t)b * seq * (n + 2 * nk) * D;
  const bf16_t *do_b = dout + (size_t)b * seq * a;
  const __amdgpu_buffer_rsrc_t rs_qkv =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(qkv_b), 0, (int)min((size_t)seq * ldq, (size_t)0x7fffffff), 0x00020000);
  const __amdgpu_buffer_rsrc_t rs_do =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(do_b), 0, (int)min((size_t)seq * ldo, (size_t)0x7fffffff), 0x00020000);
  // lse and delta of this sequence, all heads: [n][seq]
  const __amdgpu_buffer_rsrc_t rs_lse =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(lse + (size_t)b * n * seq), 0, n * seq * 4, 0x00020000);
  const __amdgpu_buffer_rsrc_t rs_del =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(delta + (size_t)b * n * seq), 0, n * seq * 4, 0x00020000);
  const int kv_wave0 = kvb * KVB + ksub * 32;
  const int kvg = kv_wave0 + lr;
  const float scale_log2 = scale * LOG2E;

  // tile k of the chunk (64 queries of one query head): Q, dO, lse, delta into ring stage k & 1
  auto issue_step = [&](int k) {
    const int u = s_begin + k, head = kh * group + u / nq_k;
    const int q0 = (first + u % nq_k) * QSTEP;
    char *st = smem_raw + OFF_RING + (k & 1) * STAGE;
    dma_tile<D, QSTEP>(rs_qkv, st, q0, seq, ldq, (unsigned)(head * D) * 2u, wave, lane);
    dma_tile<D, QSTEP>(rs_do, st + Q_TILE, q0, seq, ldo, (unsigned)(head * D) * 2u, wave, lane);
    if (wave < 2) {   // one 4-byte-per-lane instruction each for the 64 lse and delta values
      const unsigned off = (unsigned)(head * seq + min(q0 + lane, seq - 1)) * 4u;
      __builtin_amdgcn_raw_ptr_buffer_load_lds(wave == 0 ? rs_lse : rs_del,
                                               (lptr_t)(smem_raw + OFF_STAT + (k & 1) * 512 + wave * 256), 4, off, 0, 0, 0);
    }
  };

  // K and V of the 128 keys: loaded once
  dma_tile<D, KVB>(rs_qkv, smem_raw + OFF_K, kvb * KVB, seq, ldq, (unsigned)(a + kh * D) * 2u, wave, lane);
  dma_tile<D, KVB>(rs_qkv, smem_raw + OFF_V, kvb * KVB, seq, ldq, (unsigned)(a + (nk + kh) * D) * 2u, wave, lane);
  issue_step(0);

  const unsigned lds0 = (unsigned)(size_t)(const __attribute__((address_space(3))) char *)smem_raw;
  const unsigned kcl = kc_lane<D>(lane);
  unsigned trl_lo, trl_hi;
  tr_lane<D>(lane, trl_lo, trl_hi);
  const unsigned k_base = lds0 + OFF_K + ksub * 32 * RB + kcl, v_base = lds0 + OFF_V + ksub * 32 * RB + kcl;

  f32x16_t dk[D / 32], dv[D / 32];
#pragma unroll
  for (int i = 0; i < D / 32; i++)
#pragma unroll
    for (int v = 0; v < 16; v++) { dk[i][v] = 0.f; dv[i][v] = 0.f; }

  for (int k = 0; k < ns; k++) {
    // every wave's loads of tile k have landed; every wave is done with tile k-1, whose stage takes tile k+1
    STP_SB();
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
    STP_SB();
    if (k + 1 < ns) issue_step(k + 1);
    const int q0 = (first + (s_begin + k) % nq_k) * QSTEP;
    const int qs0 = q0 + 32 * qhalf;                        // this wave's 32 queries of the step
    const bool active = !causal || qs0 + 31 >= kv_wave0;    // some query sees some key of the wave
    if (!active) continue;
    const unsigned stage = lds0 + OFF_RING + (k & 1) * STAGE;
    const unsigned q_kc = stage + qhalf * 32 * RB + kcl, o_kc = q_kc + Q_TILE;
    const unsigned q_lo = stage + qhalf * 32 * RB + trl_lo, q_hi = stage + qhalf * 32 * RB + trl_hi;
    const unsigned o_lo = q_lo + Q_TILE, o_hi = q_hi + Q_TILE;
    const float *s_lse = reinterpret_cast<const float *>(smem_raw + OFF_STAT + (k & 1) * 512) + 32 * qhalf;
    const float *s_del = s_lse + 64;

    // ---- S = Q K^T and dP = dO V^T for 32 queries x 32 keys
    f32x16_t sacc, pacc;
#pragma unroll
    for (int v = 0; v < 16; v++) { sacc[v] = 0.f; pacc[v] = 0.f; }
    u32x4_t fa[4], fb[4];
#define STP_SP(buf, acc) do {                                                                                                   \
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, buf[0]), __builtin_bit_cast(bf16x8_t, buf[2]), acc, 0, 0, 0); \
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, buf[1]), __builtin_bit_cast(bf16x8_t, buf[3]), acc, 0, 0, 0); \
      STP_SB(); } while (0)
#define STP_RD_S(buf, SP) do { read_kc2<D, 0, SP>(buf[0], buf[1], q_kc); read_kc2<D, 0, SP>(buf[2], buf[3], k_base); } while (0)
#define STP_RD_P(buf, SP) do { read_kc2<D, 0, SP>(buf[0], buf[1], o_kc); read_kc2<D, 0, SP>(buf[2], buf[3], v_base); } while (0)
#define STP_RD_T(buf, lo, hi, T) do {                                                                        \
      buf[0] = read_tr<D, 16 * T>(lo, hi, 0); buf[1] = read_tr<D, 16 * T>(lo, hi, 1);                        \
      if constexpr (D == 128) { buf[2] = read_tr<D, 16 * T>(lo, hi, 2); buf[3] = read_tr<D, 16 * T>(lo, hi, 3); } } while (0)
    constexpr int TR_READS = 2 * (D / 32);
    STP_RD_S(fa, 0);
    STP_RD_P(fb, 0); lds_wait<4>(); lds_tie(fa); STP_SP(fa, sacc);
    STP_RD_S(fa, 1); lds_wait<4>(); lds_tie(fb); STP_SP(fb, pacc);
    if constexpr (D == 128) {
      STP_RD_P(fb, 1); lds_wait<4>(); lds_tie(fa); STP_SP(fa, sacc);
      STP_RD_S(fa, 2); lds_wait<4>(); lds_tie(fb); STP_SP(fb, pacc);
      STP_RD_P(fb, 2); lds_wait<4>(); lds_tie(fa); STP_SP(fa, sacc);
      STP_RD_S(fa, 3); lds_wait<4>(); lds_tie(fb); STP_SP(fb, pacc);
      STP_RD_P(fb, 3); lds_wait<4>(); lds_tie(fa); STP_SP(fa, sacc);
    } else {
      STP_RD_P(fb, 1); lds_wait<4>(); lds_tie(fa); STP_SP(fa, sacc);
    }
    STP_RD_T(fa, o_lo, o_hi, 0); lds_wait<TR_READS>(); lds_tie(fb); STP_SP(fb, pacc);   // first dO^T fragments ride through the vector phase

    // ---- P = exp(S - L), dS = P o (dP - delta); accumulator v of lane l: query qs0 + 8*(v/4) + 4*(l/32) + v%4, key kv_wave0 + l%32
    bf16x8_t pf[2], sf[2];
    auto vector_phase = [&](auto masked) {
      constexpr bool MASK = decltype(masked)::value;
#pragma unroll
      for (int j = 0; j < 4; j++) {
        const f32x4_t L4 = *reinterpret_cast<const f32x4_t *>(s_lse + 8 * j + 4 * lg);
        const f32x4_t D4 = *reinterpret_cast<const f32x4_t *>(s_del + 8 * j + 4 * lg);
#pragma unroll
        for (int r = 0; r < 4; r++) {
          const int v = 4 * j + r;
          float p = __builtin_amdgcn_exp2f(fmaf(sacc[v], scale_log2, -L4[r] * LOG2E));
          if constexpr (MASK) {
            const int qi = qs0 + 8 * j + 4 * lg + r;
            p = ((causal && qi < kvg) || qi >= seq) ? 0.f : p;
          }
          const float ds = p * (pacc[v] - D4[r]);
          pf[j >> 1][4 * (j & 1) + r] = (bf16_t)p;
          sf[j >> 1][4 * (j & 1) + r] = (bf16_t)ds;
        }
      }
    };
    if ((causal && qs0 < kv_wave0 + 31) || qs0 + 32 > seq) vector_phase(std::true_type{});
    else vector_phase(std::false_type{});
    STP_SB();

    // ---- dV^T[d, kv] += dO^T P ; dK^T[d, kv] += Q^T dS   (k = the 32 queries, two 16-steps)
#define STP_ACC(buf, acc, bop) do {                                                                                             \
      _Pragma("unroll") for (int db = 0; db < D / 32; db++)                                                                      \
        acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, buf[db]), bop, acc[db], 0, 0, 0);         \
      STP_SB(); } while (0)
    STP_RD_T(fb, q_lo, q_hi, 0); lds_wait<TR_READS>(); lds_tie(fa); STP_ACC(fa, dv, pf[0]);
    STP_RD_T(fa, o_lo, o_hi, 1); lds_wait<TR_READS>(); lds_tie(fb); STP_ACC(fb, dk, sf[0]);
    STP_RD_T(fb, q_lo, q_hi, 1); lds_wait<TR_READS>(); lds_tie(fa); STP_ACC(fa, dv, pf[1]);
    lds_wait<0>(); lds_tie(fb); STP_ACC(fb, dk, sf[1]);
#undef STP_SP
#undef STP_RD_S
#undef STP_RD_P
#undef STP_RD_T
#undef STP_ACC
  }
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
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
  if (qhalf == 0 && kvg < seq && group * nq_k <= chunk_steps) {
    // the key block has this one chunk: its rows are final and go to dK (scaled) and dV directly; the combine
    // kernel leaves them alone
    typedef bf16_t bf16x4_t __attribute__((ext_vector_type(4)));
    bf16_t *dkp = dqkv + ((size_t)b * seq + kvg) * ((size_t)(n + 2 * nk) * D) + (n + kh) * D;
    bf16_t *dvp = dkp + nk * D;
#pragma unroll
    for (int i = 0; i < D / 32; i++)
#pragma unroll
      for (int j = 0; j < 4; j++) {
        bf16x4_t wk, wv;
#pragma unroll
        for (int r = 0; r < 4; r++) {
          const int v = 4 * j + r;
          wk[r] = (bf16_t)((dk[i][v] + red[(ksub * D + i * 16 + v) * 64 + lane]) * scale);
          wv[r] = (bf16_t)(dv[i][v] + red[(ksub * D + D / 2 + i * 16 + v) * 64 + lane]);
        }
        *reinterpret_cast<bf16x4_t *>(dkp + 32 * i + 8 * j + 4 * lg) = wk;
        *reinterpret_cast<bf16x4_t *>(dvp + 32 * i + 8 * j + 4 * lg) = wv;
      }
  } else if (qhalf == 0 && kvg < seq) {
    const int nkvb = (seq + KVB - 1) / KVB;
    const size_t piece = (((size_t)b * nk + kh) * nkvb + kvb) * max_chunks + chunk;
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

// One workgroup per (key block, chunk): from the launch's work order (grid = heads x items), or, without one,
// from a grid of blocks x chunks x heads (key block 0 owns the most chunks and comes first).
template <int D>
__global__ __launch_bounds__(512) void attn_bwd_dkv_kernel(const bf16_t *__restrict__ qkv, const bf16_t *__restrict__ dout,
                                                           const float *__restrict__ lse, const float *__restrict__ delta,
                                                           float *__restrict__ part, bf16_t *__restrict__ dqkv, int seq, int n, int nk,
                                                           int causal, int max_chunks, int chunk_steps, float scale, int n_items,
                                                           stp_attn_order ord) {
  const int item = n_items ? ord.item[blockIdx.y] : 0;
  const int kvb = n_items ? (item & 0xfff) : (int)blockIdx.x, chunk = n_items ? (item >> 12) : (int)blockIdx.y;
  const int bz = n_items ? blockIdx.x : blockIdx.z;
  dkv_body<D>(qkv, dout, lse, delta, part, dqkv, seq, n, nk, causal, max_chunks, chunk_steps, scale, kvb, chunk, bz);
}

// dK = scale * sum_c, dV = sum_c over the chunks of a key block (fixed order).  One thread per 8 columns of a key row.
template <int D>
__global__ __launch_bounds__(256) void attn_bwd_dkv_combine_kernel(const float *__restrict__ part, bf16_t *__restrict__ dqkv,
                                                                   int seq, int n, int nk, int mbsz, int causal, int max_chunks,
                                                                   int chunk_steps, float scale, int kv_end) {
  const size_t idx = blockIdx.x * (size_t)256 + threadIdx.x;
  constexpr int CPR = D / 8;
  // key rows from kv_end on belong to one-chunk blocks, which the main kernel finished
  if (idx >= (size_t)mbsz * nk * kv_end * CPR) return;
  const int c8 = (idx % CPR) * 8;
  const size_t row = idx / CPR;
  const int kv = row % kv_end, kh = (row / kv_end) % nk, b = row / ((size_t)kv_end * nk);
  const int kvb = kv / KVB, kloc = kv % KVB;
  const int nkvb = (seq + KVB - 1) / KVB, nq = (seq + QSTEP - 1) / QSTEP;
  const int nch = ((n / nk) * (nq - dkv_first_step(kvb, causal)) + chunk_steps - 1) / chunk_steps;
  if (nch <= 1) return;
  const float *p0 = part + ((((size_t)b * nk + kh) * nkvb + kvb) * max_chunks) * (size_t)(2 * KVB * D) + (size_t)kloc * D + c8;
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
  bf16_t *dkp = dqkv + ((size_t)b * seq + kv) * ((size_t)(n + 2 * nk) * D) + (n + kh) * D + c8;
  Vec8<bf16_t>::store(dkp, sk);
  Vec8<bf16_t>::store(dkp + nk * D, sv);
}

// ---------------------------------------------------------------------------------------------
// dQ partials.  piece layout: dQ [128][D] fp32 (unscaled)
// ---------------------------------------------------------------------------------------------
template <int D>
__device__ __forceinline__ void dq_body(const bf16_t *__restrict__ qkv, const bf16_t *__restrict__ dout,
                                        const float *__restrict__ lse, const float *__restrict__ delta,
                                        float *__restrict__ part, bf16_t *__restrict__ dqkv, int seq, int n, int nk, int causal,
                                        int max_chunks, int chunk_steps, float scale, int qb, int chunk, int bz) {
  using G = BG<D>;
  constexpr int RB = G::RB;
  constexpr int KV_TILE = KVB * RB, STAGE = 2 * KV_TILE;      // LDS: ring of two stages { K [128][D], V [128][D] }
  extern __shared__ __attribute__((aligned(1024))) char smem_raw[];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lr = lane & 31, lg = lane >> 5;
  const int qsub = wave & 3, half = wave >> 2;
  const int nqblk = (seq + 127) / 128;
  const int head = bz % n, b = bz / n;
  const int nsteps = dq_steps(qb, seq, causal);
  const int s_begin = chunk * chunk_steps, s_end = min(nsteps, s_begin + chunk_steps);
  if (s_begin >= nsteps) return;
  const int ns = s_end - s_begin;

  const int a = n * D;
  const size_t ld = (size_t)(n + 2 * nk) * D;            // a qkv row: n Q heads, nk K heads, nk V heads
  const unsigned ldq = (unsigned)ld * 2u;
  const int kcol = a + (head / (n / nk)) * D, vcol = kcol + nk * D;   // this head's key / value head
  const bf16_t *qkv_b = qkv + (size_t)b * seq * ld;
  const bf16_t *qbase = qkv_b + head * D;
  const bf16_t *dobase = dout + (size_t)b * seq * a + head * D;
  const __amdgpu_buffer_rsrc_t rs_qkv =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(qkv_b), 0, (int)min((size_t)seq * ldq, (size_t)0x7fffffff), 0x00020000);
  auto issue_step = [&](int k) {
    char *st = smem_raw + (k & 1) * STAGE;
    dma_tile<D, KVB>(rs_qkv, st, (s_begin + k) * KVB, seq, ldq, (unsigned)kcol * 2u, wave, lane);
    dma_tile<D, KVB>(rs_qkv, st + KV_TILE, (s_begin + k) * KVB, seq, ldq, (unsigned)vcol * 2u, wave, lane);
  };
  issue_step(0);

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

  const unsigned lds0 = (unsigned)(size_t)(const __attribute__((address_space(3))) char *)smem_raw;
  const unsigned kcl = kc_lane<D>(lane);
  unsigned trl_lo, trl_hi;
  tr_lane<D>(lane, trl_lo, trl_hi);

  for (int k = 0; k < ns; k++) {
    // every wave's loads of tile k have landed; every wave is done with tile k-1, whose stage takes tile k+1
    STP_SB();
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
    STP_SB();
    if (k + 1 < ns) issue_step(k + 1);
    const int kv0 = (s_begin + k) * KVB + 64 * half;          // this wave's 64 keys of the step
    const bool active = kv0 < seq && (!causal || kv0 <= q_wave0 + 31);
    if (!active) continue;
    const bool need_mask = (causal && kv0 + 63 > q_wave0) || (kv0 + 64 > seq);
    const unsigned stage = lds0 + (k & 1) * STAGE + 64 * half * RB;
    const unsigned k_kc = stage + kcl, v_kc = k_kc + KV_TILE;
    const unsigned k_lo = stage + trl_lo, k_hi = stage + trl_hi;

    u32x4_t fa[4], fb[4];
    f32x16_t sacc, pacc;
    bf16x8_t sf[2];
    constexpr int TR_READS = 2 * (D / 32);
    // four 16-byte fragments (k-steps 4*SG .. 4*SG+3) of the 32 tile rows from ROW0
#define STP_RD4(buf, base, ROW0, SG) do { read_kc2<D, ROW0, 2 * (SG)>(buf[0], buf[1], base); read_kc2<D, ROW0, 2 * (SG) + 1>(buf[2], buf[3], base); } while (0)
#define STP_MF4(buf, acc, bop, SG) do {                                                                                          \
      _Pragma("unroll") for (int i = 0; i < 4; i++)                                                                               \
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, buf[i]), bop[4 * (SG) + i], acc, 0, 0, 0);     \
      STP_SB(); } while (0)
#define STP_RD_T(buf, R0) do {                                                                               \
      buf[0] = read_tr<D, R0>(k_lo, k_hi, 0); buf[1] = read_tr<D, R0>(k_lo, k_hi, 1);                        \
      if constexpr (D == 128) { buf[2] = read_tr<D, R0>(k_lo, k_hi, 2); buf[3] = read_tr<D, R0>(k_lo, k_hi, 3); } } while (0)
#define STP_ACC(buf, bop) do {                                                                                                   \
      _Pragma("unroll") for (int db = 0; db < D / 32; db++)                                                                      \
        dq[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, buf[db]), bop, dq[db], 0, 0, 0);           \
      STP_SB(); } while (0)
    // accumulator v of lane l: key kv0 + 32*ks + 8*(v/4) + 4*(l/32) + v%4, query q_wave0 + l%32
    auto vector_phase = [&](int ks, auto masked) {
      constexpr bool MASK = decltype(masked)::value;
#pragma unroll
      for (int v = 0; v < 16; v++) {
        float p = __builtin_amdgcn_exp2f(fmaf(sacc[v], scale_log2, -L2));
        if constexpr (MASK) {
          const int kv = kv0 + 32 * ks + 8 * (v >> 2) + 4 * lg + (v & 3);
          p = ((causal && kv > qg) || kv >= seq) ? 0.f : p;
        }
        sf[v >> 3][v & 7] = (bf16_t)(p * (pacc[v] - Dl));
      }
    };
    // one 32-key sub-block: S^T = K Q^T, dP^T = V dO^T, dS^T, dQ^T += K^T dS^T.  On entry fa holds (or is receiving)
    // the first four K fragments; NEXT names what to prefetch behind the last MFMA group.
#define STP_SUBBLOCK(KS, NEXT)                                                                                                    \
    do {                                                                                                                          \
      _Pragma("unroll") for (int v = 0; v < 16; v++) { sacc[v] = 0.f; pacc[v] = 0.f; }                                            \
      if constexpr (D == 128) {                                                                                                   \
        STP_RD4(fb, k_kc, 32 * KS, 1); lds_wait<4>(); lds_tie(fa); STP_MF4(fa, sacc, qf, 0);                                      \
        STP_RD4(fa, v_kc, 32 * KS, 0); lds_wait<4>(); lds_tie(fb); STP_MF4(fb, sacc, qf, 1);                                      \
        STP_RD4(fb, v_kc, 32 * KS, 1); lds_wait<4>(); lds_tie(fa); STP_MF4(fa, pacc, of, 0);                                      \
        STP_RD_T(fa, 32 * KS); lds_wait<TR_READS>(); lds_tie(fb); STP_MF4(fb, pacc, of, 1);                                       \
      } else {                                                                                                                    \
        STP_RD4(fb, v_kc, 32 * KS, 0); lds_wait<4>(); lds_tie(fa); STP_MF4(fa, sacc, qf, 0);                                      \
        STP_RD_T(fa, 32 * KS); lds_wait<TR_READS>(); lds_tie(fb); STP_MF4(fb, pacc, of, 0);                                       \
      }                                                                                                                           \
      if (need_mask) vector_phase(KS, std::true_type{}); else vector_phase(KS, std::false_type{});                                \
      STP_SB();                                                                                                                   \
      STP_RD_T(fb, 32 * KS + 16); lds_wait<TR_READS>(); lds_tie(fa); STP_ACC(fa, sf[0]);                                          \
      NEXT;                                                                                                                       \
      STP_ACC(fb, sf[1]);                                                                                                         \
    } while (0)
    STP_RD4(fa, k_kc, 0, 0);
    STP_SUBBLOCK(0, STP_RD4(fa, k_kc, 32, 0); lds_wait<4>(); lds_tie(fb));
    STP_SUBBLOCK(1, lds_wait<0>(); lds_tie(fb));
#undef STP_RD4
#undef STP_MF4
#undef STP_RD_T
#undef STP_ACC
#undef STP_SUBBLOCK
  }
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
  float *red = reinterpret_cast<float *>(smem_raw);        // [4][D/2][64]
  if (half == 1) {
#pragma unroll
    for (int i = 0; i < D / 32; i++)
#pragma unroll
      for (int v = 0; v < 16; v++) red[(qsub * (D / 2) + i * 16 + v) * 64 + lane] = dq[i][v];
  }
  __syncthreads();
  if (half == 0 && qg < seq && nsteps <= chunk_steps) {
    // the query block has this one chunk: its rows are final and go to dQ (scaled) directly
    typedef bf16_t bf16x4_t __attribute__((ext_vector_type(4)));
    bf16_t *dqp = dqkv + ((size_t)b * seq + qg) * ((size_t)(n + 2 * nk) * D) + head * D;
#pragma unroll
    for (int i = 0; i < D / 32; i++)
#pragma unroll
      for (int j = 0; j < 4; j++) {
        bf16x4_t w;
#pragma unroll
        for (int r = 0; r < 4; r++) {
          const int v = 4 * j + r;
          w[r] = (bf16_t)((dq[i][v] + red[(qsub * (D / 2) + i * 16 + v) * 64 + lane]) * scale);
        }
        *reinterpret_cast<bf16x4_t *>(dqp + 32 * i + 8 * j + 4 * lg) = w;
      }
  } else if (half == 0 && qg < seq) {
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

// One workgroup per (query block, chunk): from the launch's work order (grid = heads x items), or, without
// one, from a grid of blocks x chunks x heads with the late query blocks, which own the most chunks, first.
template <int D>
__global__ __launch_bounds__(512) void attn_bwd_dq_kernel(const bf16_t *__restrict__ qkv, const bf16_t *__restrict__ dout,
                                                          const float *__restrict__ lse, const float *__restrict__ delta,
                                                          float *__restrict__ part, bf16_t *__restrict__ dqkv, int seq, int n, int nk,
                                                          int causal, int max_chunks, int chunk_steps, float scale, int n_items,
                                                          stp_attn_order ord) {
  const int nqblk = (seq + 127) / 128;
  const int item = n_items ? ord.item[blockIdx.y] : 0;
  const int qb = n_items ? (item & 0xfff) : nqblk - 1 - (int)blockIdx.x;
  const int chunk = n_items ? (item >> 12) : (int)blockIdx.y;
  const int bz = n_items ? blockIdx.x : blockIdx.z;
  dq_body<D>(qkv, dout, lse, delta, part, dqkv, seq, n, nk, causal, max_chunks, chunk_steps, scale, qb, chunk, bz);
}

// Both kernels in one launch (same number of query and key / value heads): a work item is a dkv or a dq
// (block, chunk) pair, item = block | chunk << 12 | (1 << 15 for dq), sorted by estimated time, longest first.
// The two kinds fill each other's idle compute units: their workgroups are few and of unequal length.
template <int D>
__global__ __launch_bounds__(512) void attn_bwd_fused_kernel(const bf16_t *__restrict__ qkv, const bf16_t *__restrict__ dout,
                                                             const float *__restrict__ lse, const float *__restrict__ delta,
                                                             float *__restrict__ part_kv, float *__restrict__ part_q,
                                                             bf16_t *__restrict__ dqkv, int seq, int n,
                                                             int nk, int causal, int mc_kv, int ch_kv, int mc_q, int ch_q, float scale,
                                                             stp_attn_order ord
#ifdef STP_ATTN_TRACE
                                                             , long long *trace
#endif
                                                             ) {
#ifdef STP_ATTN_TRACE
  const long long tr0 = wall_clock64();
#endif
  const int item = ord.item[blockIdx.y];
  const int block = item & 0xfff, chunk = (item >> 12) & 7, bz = blockIdx.x;
  if (item & 0x8000) dq_body<D>(qkv, dout, lse, delta, part_q, dqkv, seq, n, nk, causal, mc_q, ch_q, scale, block, chunk, bz);
  else dkv_body<D>(qkv, dout, lse, delta, part_kv, dqkv, seq, n, nk, causal, mc_kv, ch_kv, scale, block, chunk, bz);
#ifdef STP_ATTN_TRACE
  if (trace) {   // per-workgroup life time: start, end, work item
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    const long long tr3 = wall_clock64();
    if (threadIdx.x == 0) {
      long long *t = trace + ((size_t)blockIdx.y * gridDim.x + blockIdx.x) * 4;
      t[0] = tr0; t[1] = tr3; t[2] = item; t[3] = 1;
    }
  }
#endif
}

template <int D>
__global__ __launch_bounds__(256) void attn_bwd_dq_combine_kernel(const float *__restrict__ part, bf16_t *__restrict__ dqkv,
                                                                  int seq, int n, int nk, int mbsz, int causal, int max_chunks,
                                                                  int chunk_steps, float scale, int q_first) {
  const size_t idx = blockIdx.x * (size_t)256 + threadIdx.x;
  constexpr int CPR = D / 8;
  const int rows = seq - q_first;           // query rows below q_first belong to one-chunk blocks, which the main kernel finished
  if (idx >= (size_t)mbsz * n * rows * CPR) return;
  const int c8 = (idx % CPR) * 8;
  const size_t row = idx / CPR;
  const int q = q_first + row % rows, head = (row / rows) % n, b = row / ((size_t)rows * n);
  const int qb = q / 128, qloc = q % 128;
  const int nqblk = (seq + 127) / 128;
  const int nch = (dq_steps(qb, seq, causal) + chunk_steps - 1) / chunk_steps;
  if (nch <= 1) return;
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
  Vec8<bf16_t>::store(dqkv + ((size_t)b * seq + q) * ((size_t)(n + 2 * nk) * D) + head * D + c8, sq);
}

// the plans of the two kernels for this shape (dkv: block x = key block x; dq: block x = query block x)
inline const stp_attn_plan *dkv_plan(stp_ctx *ctx, const stp_layer_desc *d) {
  const int nkvb = (d->seq + KVB - 1) / KVB, nq = (d->seq + QSTEP - 1) / QSTEP;
  std::vector<int> steps(nkvb);
  const int group = d->heads_local / stp_kv_heads(d);     // a key block runs over the steps of its whole head group
  for (int x = 0; x < nkvb; x++) steps[x] = group * (nq - dkv_first_step(x, d->causal));
  return stp_attn_plan_get(ctx, 1, d, nkvb, steps.data(), stp_kv_heads(d) * d->mbsz);
}
inline const stp_attn_plan *dq_plan(stp_ctx *ctx, const stp_layer_desc *d) {
  const int nqb = (d->seq + 127) / 128;
  std::vector<int> steps(nqb);
  for (int x = 0; x < nqb; x++) steps[x] = dq_steps(x, d->seq, d->causal);
  return stp_attn_plan_get(ctx, 2, d, nqb, steps.data(), d->heads_local * d->mbsz);
}

// The merged work order of the fused launch: the (block, chunk) pairs of both kernels, sorted by the plan's
// estimate of their time, longest first (ties keep dkv before dq and each kernel's own order).
const stp_attn_plan *fused_plan(stp_ctx *ctx, const stp_layer_desc *d, const stp_attn_plan &pkv, const stp_attn_plan &pq) {
  const int key[8] = {4 + (ctx && ctx->concurrent ? 16 : 0), d->seq, d->causal, d->heads_local, stp_kv_heads(d), d->mbsz, d->head_dim, 0};
  bool hit;
  stp_attn_plan *p = stp_attn_plan_slot(ctx, key, &hit);
  if (hit) return p;
  const int nq = (d->seq + QSTEP - 1) / QSTEP, group = d->heads_local / stp_kv_heads(d);
  struct Item { double cost; uint16_t item; };
  std::vector<Item> items;
  for (int i = 0; i < pkv.n_items; i++) {
    const int x = pkv.order.item[i] & 0xfff, k = pkv.order.item[i] >> 12;
    const int steps = group * (nq - dkv_first_step(x, d->causal));
    items.push_back({stp_attn_item_cost(1, std::min(pkv.chunk_steps, steps - k * pkv.chunk_steps)), pkv.order.item[i]});
  }
  for (int i = 0; i < pq.n_items; i++) {
    const int x = pq.order.item[i] & 0xfff, k = pq.order.item[i] >> 12;
    const int steps = dq_steps(x, d->seq, d->causal);
    items.push_back({stp_attn_item_cost(2, std::min(pq.chunk_steps, steps - k * pq.chunk_steps)), (uint16_t)(pq.order.item[i] | 0x8000)});
  }
  std::stable_sort(items.begin(), items.end(), [](const Item &u, const Item &v) { return u.cost > v.cost; });
  p->chunk_steps = 0;
  p->max_chunks = 0;
  p->n_items = (int)items.size();
  for (size_t i = 0; i < items.size(); i++) p->order.item[i] = items[i].item;
  return p;
}

template <int D>
int launch_bwd(stp_ctx *ctx, const stp_layer_desc *d, const void *qkv, const float *lse, const void *dout, const float *delta,
               void *dqkv, float *ws, size_t ws_bytes, hipStream_t s) {
  using G = BG<D>;
  constexpr size_t smem_kv = (size_t)(2 * KVB + 4 * QSTEP) * G::RB + 2 * 512;   // K, V, ring of {Q, dO}, ring of {lse, delta}
  constexpr size_t smem_q = (size_t)4 * KVB * G::RB;                              // ring of {K, V}
  constexpr size_t smem_f = smem_kv > smem_q ? smem_kv : smem_q;
  static_assert(smem_kv <= 160 * 1024 && smem_kv >= (size_t)4 * D * 64 * sizeof(float), "dkv LDS budget");
  static_assert(smem_q <= 160 * 1024 && smem_q >= (size_t)4 * (D / 2) * 64 * sizeof(float), "dq LDS budget");
  if ((size_t)d->seq * stp_qkv_width(d) * sizeof(bf16_t) > (size_t)0x7fffffff)
    return stp_fail(ctx, STP_ESHAPE, "attention backward: one sequence of QKV must span less than 2 GiB%s");
  auto kkv = attn_bwd_dkv_kernel<D>;
  auto kq = attn_bwd_dq_kernel<D>;
  auto kf = attn_bwd_fused_kernel<D>;
  static bool attr_set = false;
  if (!attr_set) {
    STP_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(kkv), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem_kv));
    STP_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(kq), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem_q));
    STP_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(kf), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem_f));
    attr_set = true;
  }
  const float scale = 1.0f / sqrtf((float)D);
  const int nkvb = (d->seq + KVB - 1) / KVB, nqb = (d->seq + 127) / 128;
  const int nk = stp_kv_heads(d);
  // copies: a later lookup may evict an earlier plan from the context's cache
  const stp_attn_plan pkv = *dkv_plan(ctx, d), pq = *dq_plan(ctx, d);
  const int ch_kv = pkv.chunk_steps, ch_q = pq.chunk_steps, mc_kv = pkv.max_chunks, mc_q = pq.max_chunks;
  const size_t bh = (size_t)d->mbsz * d->heads_local, bk = (size_t)d->mbsz * nk;
  // the partials of the two kernels lie one behind the other: with equal head counts both run in one launch
  const size_t need_kv = stp_align_up(bk * nkvb * mc_kv * 2 * KVB * D * sizeof(float), 256), need_q = bh * nqb * mc_q * 128 * D * sizeof(float);
  const size_t need = need_kv + need_q;
  if (!ws || ws_bytes < need)
    return stp_fail(ctx, STP_ENOSPACE, "attention backward: workspace lane too small%s (need %ld bytes)", "", (long)need);
  float *ws_kv = ws, *ws_q = ws + need_kv / sizeof(float);
  const bool fused = bk == bh && pkv.n_items && pq.n_items && pkv.n_items + pq.n_items <= STP_ATTN_ORDER_CAP;
  if (fused) {
    const stp_attn_plan *pf = fused_plan(ctx, d, pkv, pq);
    hipLaunchKernelGGL(kf, dim3((unsigned)bh, pf->n_items), dim3(512), smem_f, s, (const bf16_t *)qkv, (const bf16_t *)dout, lse, delta,
                       ws_kv, ws_q, (bf16_t *)dqkv, d->seq, d->heads_local, nk, d->causal, mc_kv, ch_kv, mc_q, ch_q, scale, pf->order
#ifdef STP_ATTN_TRACE
                       , getenv("STP_TRACE_PTR") ? (long long *)strtoull(getenv("STP_TRACE_PTR"), nullptr, 0) : (long long *)nullptr
#endif
                       );
    STP_LAUNCH_CHECK(ctx);
  } else {
    hipLaunchKernelGGL(kkv, pkv.n_items ? dim3((unsigned)bk, pkv.n_items) : dim3(nkvb, mc_kv, (unsigned)bk), dim3(512), smem_kv, s,
                       (const bf16_t *)qkv, (const bf16_t *)dout, lse, delta, ws_kv, (bf16_t *)dqkv, d->seq, d->heads_local, nk, d->causal, mc_kv,
                       ch_kv, scale, pkv.n_items, pkv.order);
    STP_LAUNCH_CHECK(ctx);
    hipLaunchKernelGGL(kq, pq.n_items ? dim3((unsigned)bh, pq.n_items) : dim3(nqb, mc_q, (unsigned)bh), dim3(512), smem_q, s,
                       (const bf16_t *)qkv, (const bf16_t *)dout, lse, delta, ws_q, (bf16_t *)dqkv, d->seq, d->heads_local, nk, d->causal, mc_q, ch_q,
                       scale, pq.n_items, pq.order);
    STP_LAUNCH_CHECK(ctx);
  }
  // Blocks with a single chunk were finished by the main kernels.  A key block's steps fall with its index (with the
  // causal mask; otherwise all are equal), a query block's rise: the combine kernels run over the other rows only.
  const int nq64 = (d->seq + QSTEP - 1) / QSTEP, group = d->heads_local / nk;
  int kvb_end = nkvb, qb_first = 0;
  while (kvb_end > 0 && group * (nq64 - dkv_first_step(kvb_end - 1, d->causal)) <= ch_kv) kvb_end--;
  while (qb_first < nqb && dq_steps(qb_first, d->seq, d->causal) <= ch_q) qb_first++;
  if (kvb_end > 0) {
    const int kv_end = std::min(d->seq, kvb_end * KVB);
    const size_t r8 = bk * kv_end * (D / 8);
    hipLaunchKernelGGL(attn_bwd_dkv_combine_kernel<D>, dim3((r8 + 255) / 256), dim3(256), 0, s, ws_kv, (bf16_t *)dqkv, d->seq,
                       d->heads_local, nk, d->mbsz, d->causal, mc_kv, ch_kv, scale, kv_end);
    STP_LAUNCH_CHECK(ctx);
  }
  if (qb_first < nqb) {
    const int q_first = qb_first * 128;
    const size_t r8 = bh * (d->seq - q_first) * (D / 8);
    hipLaunchKernelGGL(attn_bwd_dq_combine_kernel<D>, dim3((r8 + 255) / 256), dim3(256), 0, s, ws_q, (bf16_t *)dqkv, d->seq,
                       d->heads_local, nk, d->mbsz, d->causal, mc_q, ch_q, scale, q_first);
    STP_LAUNCH_CHECK(ctx);
  }
  return STP_OK;
}

}  // namespace

const stp_attn_plan *stp_attn_bwd_plan_for(stp_ctx *ctx, const stp_layer_desc *d, int kind) {
  return kind == 1 ? dkv_plan(ctx, d) : dq_plan(ctx, d);
}

size_t stp_attn_bwd_ws_bytes(const stp_layer_desc *d) {
  const int nkvb = (d->seq + KVB - 1) / KVB, nqb = (d->seq + 127) / 128;
  const int nk = stp_kv_heads(d);
  const size_t bh = (size_t)d->mbsz * d->heads_local, bk = (size_t)d->mbsz * nk;
  const size_t need_kv = stp_align_up(bk * nkvb * dkv_plan(nullptr, d)->max_chunks * 2 * KVB * d->head_dim * sizeof(float), 256);
  const size_t need_q = bh * nqb * dq_plan(nullptr, d)->max_chunks * 128 * d->head_dim * sizeof(float);
  return need_kv + need_q;
}

int stp_launch_attn_bwd_bf16(stp_ctx *ctx, const stp_layer_desc *d, const void *qkv, const void *out, const float *lse,
                             const void *dout, float *delta, void *dqkv, float *ws, size_t ws_bytes, hipStream_t s) {
  int rc = stp_launch_rowdot(ctx, d, dout, out, delta, s);
  if (rc != STP_OK) return rc;
  if (d->head_dim == 128) return launch_bwd<128>(ctx, d, qkv, lse, dout, delta, dqkv, ws, ws_bytes, s);
  if (d->head_dim == 64) return launch_bwd<64>(ctx, d, qkv, lse, dout, delta, dqkv, ws, ws_bytes, s);
  return stp_fail(ctx, STP_ESHAPE, "bf16 attention needs head_dim 64 or 128%s");
}

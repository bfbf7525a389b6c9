// Tiled attention forward for bf16 on the CDNA4 matrix cores ("Attention(.)" of Eq. 1:
// the attention core of one TP rank, no communication).
//
// Work decomposition.  A workgroup owns 128 query rows of one (sequence, head) and ONE CHUNK of up
// to 1024 keys; chunks of the same query block are merged afterwards by a small combine kernel
// (fixed order, deterministic).  Cutting the key range into chunks turns the causal triangle into
// ~3 pieces of similar size per compute unit instead of 192 workgroups whose length varies 1..96.
// Inside a workgroup 8 waves run as 4 query sub-tiles (32 rows) x 2 key halves: per 128-key step
// waves 0-3 take keys 0..63 and waves 4-7 keys 64..127, so every SIMD holds two waves and one
// wave's softmax arithmetic overlaps the other's MFMAs.  The two halves are merged through LDS.
//
// Per wave the kernel works on the TRANSPOSED score tile, S^T = K Q^T: with the 32x32x16 MFMA the
// accumulator of lane l then holds column q = l % 32, i.e. every softmax statistic (running max,
// running sum, rescale factor) is a per-lane scalar and a row reduction is an in-lane loop plus one
// cross-half shuffle.  The probabilities are already in the register layout the next MFMA wants for
// its B operand (O^T += V^T P^T), so P never touches LDS.  V^T fragments come from the V tile as it
// lies in memory ([kv][d]) through the transposing LDS read.
//   K tile  : LDS [128][D + 8]   16-byte fragment reads
//   V tile  : LDS [128][D + 32]  ds_read_b64_tr_b16 fragment reads
// Both are double-buffered through registers (next step's loads in flight during the MFMAs of the
// current one).
#include "common.h"

namespace {

constexpr int QB = 128;    // query rows per workgroup
constexpr int KSTEP = 128; // keys per step (64 per wave half)
constexpr int CH2 = 8;     // steps per chunk (1024 keys)
constexpr float LN2 = 0.69314718055994531f;

typedef s16x4_t __attribute__((address_space(3))) * lds_s16x4_ptr;

template <int D> struct AttnGeom {
  static constexpr int kp = D + 8;    // K tile pitch (elements)
  static constexpr int vp = D + 32;   // V tile pitch
  static constexpr int k_elems = KSTEP * kp;
  static constexpr int v_elems = KSTEP * vp;
  static constexpr int nld = KSTEP * D / 8 / 512;  // 16-byte chunks per thread per tile
  static constexpr int piece_floats = QB * D + 2 * QB;   // partial O, then m, then l
};

// 128 x D tile, 512 threads: registers <- global (rows clamped to seq-1; keys past the end are masked later)
template <int D, int NLD>
__device__ __forceinline__ void tile_load(uint4 (&r)[NLD], const bf16_t *__restrict__ base, size_t ld, int row0, int seq, int tid) {
  static_assert(NLD == KSTEP * D / 8 / 512, "register count");
#pragma unroll
  for (int i = 0; i < NLD; i++) {
    int q = tid + 512 * i;
    int rr = q / (D / 8), c = (q % (D / 8)) * 8;
    int row = min(row0 + rr, seq - 1);
    const uint4 v = *reinterpret_cast<const uint4 *>(base + (size_t)row * ld + c);
    r[i].x = v.x; r[i].y = v.y; r[i].z = v.z; r[i].w = v.w;
  }
}
template <int D, int P, int NLD>
__device__ __forceinline__ void tile_store(const uint4 (&r)[NLD], bf16_t *tile, int tid) {
#pragma unroll
  for (int i = 0; i < NLD; i++) {
    int q = tid + 512 * i;
    int rr = q / (D / 8), c = (q % (D / 8)) * 8;
    uint4 v;   // component-wise copy: a whole-struct copy keeps the register array in scratch memory
    v.x = r[i].x; v.y = r[i].y; v.z = r[i].z; v.w = r[i].w;
    *reinterpret_cast<uint4 *>(tile + rr * P + c) = v;
  }
}

// number of 128-key steps a query block needs
__host__ __device__ inline int attn_steps(int qb, int seq, int causal) {
  int kv_end = causal ? (seq < qb * QB + QB ? seq : qb * QB + QB) : seq;
  return (kv_end + KSTEP - 1) / KSTEP;
}

template <int D>
__global__ __launch_bounds__(512) void attn_fwd_bf16_kernel(const bf16_t *__restrict__ qkv, float *__restrict__ part, int seq,
                                                            int n, int causal, int max_chunks, float scale_log2) {
  using G = AttnGeom<D>;
  extern __shared__ __attribute__((aligned(16))) char smem_raw[];
  constexpr int STAGE = G::k_elems + G::v_elems;
  bf16_t *const sbase = reinterpret_cast<bf16_t *>(smem_raw);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lr = lane & 31, lg = lane >> 5;
  const int qsub = wave & 3, half = wave >> 2;
  const int nqb = (seq + QB - 1) / QB;
  const int qb = nqb - 1 - blockIdx.x;              // late query blocks own the most chunks: start them first
  const int chunk = blockIdx.y;
  const int head = blockIdx.z % n, b = blockIdx.z / n;
  const int nsteps = attn_steps(qb, seq, causal);
  const int s_begin = chunk * CH2, s_end = min(nsteps, s_begin + CH2);
  if (s_begin >= nsteps) return;

  const int a = n * D;
  const size_t ld = 3 * (size_t)a;
  const bf16_t *base = qkv + (size_t)b * seq * ld + head * D;  // Q of this head; K at +a, V at +2a
  const int q_wave0 = qb * QB + qsub * 32;
  const int qg = q_wave0 + lr;                  // this lane's query row
  const int q_ld = min(qg, seq - 1);            // clamp so that tail lanes read valid memory

  // Q fragments: B operand, lane supplies row q, k = d index 16*s + 8*lg .. +7
  bf16x8_t qf[D / 16];
#pragma unroll
  for (int s = 0; s < D / 16; s++)
    qf[s] = *reinterpret_cast<const bf16x8_t *>(base + (size_t)q_ld * ld + 16 * s + 8 * lg);

  f32x16_t o[D / 32];
#pragma unroll
  for (int i = 0; i < D / 32; i++)
#pragma unroll
    for (int v = 0; v < 16; v++) o[i][v] = 0.f;
  float m = -INFINITY, l = 0.f;
  const bf16_t *kbase = base + a;

  uint4 rk[G::nld], rv[G::nld];
  tile_load<D>(rk, kbase, ld, s_begin * KSTEP, seq, tid);
  tile_load<D>(rv, kbase + a, ld, s_begin * KSTEP, seq, tid);
  tile_store<D, G::kp>(rk, sbase, tid);
  tile_store<D, G::vp>(rv, sbase + G::k_elems, tid);
  __syncthreads();

  for (int st = s_begin; st < s_end; st++) {
    const int cur = (st - s_begin) & 1;
    const bf16_t *ks_cur = sbase + cur * STAGE + half * 64 * G::kp;
    const bf16_t *vs_cur = sbase + cur * STAGE + G::k_elems + half * 64 * G::vp;
    const int kv0 = st * KSTEP + half * 64;       // first key of this wave's 64-key block
    if (st + 1 < s_end) {
      tile_load<D>(rk, kbase, ld, (st + 1) * KSTEP, seq, tid);
      tile_load<D>(rv, kbase + a, ld, (st + 1) * KSTEP, seq, tid);
    }

    // wave-uniform skip: all of this wave's queries precede the key block, or the block is past the end
    const bool active = kv0 < seq && (!causal || kv0 <= q_wave0 + 31);
    if (active) {
      // ---- S^T[kv, q] = K Q^T for the two 32-key sub-blocks (named accumulators: an array of vectors
      //      would be demoted to scratch memory)
      auto scores = [&](int jb) {
        f32x16_t acc;
#pragma unroll
        for (int v = 0; v < 16; v++) acc[v] = 0.f;
#pragma unroll
        for (int s = 0; s < D / 16; s++) {
          bf16x8_t kf = *reinterpret_cast<const bf16x8_t *>(ks_cur + (32 * jb + lr) * G::kp + 16 * s + 8 * lg);
          acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[s], acc, 0, 0, 0);
        }
        return acc;
      };
      f32x16_t sc0 = scores(0), sc1 = scores(1);
      // ---- online softmax in the log2 domain; accumulator v of lane l is key
      //      kv0 + 32*jb + 8*(v/4) + 4*(l/32) + v%4, query l%32
      const bool need_mask = (causal && kv0 + 63 > q_wave0) || (kv0 + 64 > seq);
      // raw scores are kept; the 1/sqrt(d) log2(e) factor is folded into the exponent's FMA
      auto mask_max = [&](f32x16_t &sc, int jb, float mx) {
#pragma unroll
        for (int v = 0; v < 16; v++) {
          if (need_mask) {
            int kv = kv0 + 32 * jb + 8 * (v >> 2) + 4 * lg + (v & 3);
            if ((causal && kv > qg) || kv >= seq) sc[v] = -INFINITY;
          }
          mx = fmaxf(mx, sc[v]);
        }
        return mx;
      };
      float mx = mask_max(sc0, 0, -INFINITY);
      mx = mask_max(sc1, 1, mx);
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64)) * scale_log2;      // scale > 0: max and scaling commute
      // Lazy rescaling: the reference m only moves when the block maximum exceeds it by more than 2^8,
      // so exponentials stay below 256 (harmless in fp32 / bf16) and the O rescale is skipped on almost
      // every block.  Softmax is invariant to the reference as long as l, O and P use the same one.
      // A query row that has seen no admissible key keeps m = -inf.
      const float m_new = (mx > m + 8.0f) ? mx : m;
      if (__builtin_amdgcn_ballot_w64(m_new != m) != 0) {
        const float corr = __builtin_amdgcn_exp2f(m - (m_new == -INFINITY ? 0.f : m_new));
        l *= corr;
#pragma unroll
        for (int i = 0; i < D / 32; i++)
#pragma unroll
          for (int v = 0; v < 16; v++) o[i][v] *= corr;
        m = m_new;
      }
      const float neg_ref = m == -INFINITY ? 0.f : -m;
      auto exp_sum = [&](f32x16_t &sc, float rs) {
#pragma unroll
        for (int v = 0; v < 16; v++) {
          float p = __builtin_amdgcn_exp2f(fmaf(sc[v], scale_log2, neg_ref));
          sc[v] = p;
          rs += p;
        }
        return rs;
      };
      float rs = exp_sum(sc0, 0.f);
      rs = exp_sum(sc1, rs);
      rs += __shfl_xor(rs, 32, 64);
      l += rs;

      // ---- O^T[d, q] += V^T P^T ; k-slot i of lane-half g in step (jb, t) is key 32*jb + 16*t + 8*(i/4) + 4*g + i%4
      auto pv = [&](const f32x16_t &sc, int jb) {
#pragma unroll
        for (int t = 0; t < 2; t++) {
          bf16x8_t pf;
#pragma unroll
          for (int i = 0; i < 8; i++) pf[i] = (bf16_t)sc[8 * t + i];
          const int krow = 32 * jb + 16 * t + 4 * lg + ((lane & 15) >> 2);
#pragma unroll
          for (int db = 0; db < D / 32; db++) {
            const bf16_t *p = vs_cur + krow * G::vp + 32 * db + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
            s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p));
            s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p + 8 * G::vp));
            s16x8_t vv = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, vv), pf, o[db], 0, 0, 0);
          }
        }
      };
      pv(sc0, 0);
      pv(sc1, 1);
    }
    if (st + 1 < s_end) {
      tile_store<D, G::kp>(rk, sbase + (cur ^ 1) * STAGE, tid);
      tile_store<D, G::vp>(rv, sbase + (cur ^ 1) * STAGE + G::k_elems, tid);
    }
    __syncthreads();
  }

  // ---- merge the two key halves (upper half -> LDS -> lower half), then write this chunk's partial:
  // O (un-normalised, relative to m), m (log2 domain), l.
  float *red = reinterpret_cast<float *>(smem_raw);            // [4][D/2][64] accumulators, then [4][2][32] m, l
  float *red_ml = red + 4 * (D / 2) * 64;
  if (half == 1) {
#pragma unroll
    for (int i = 0; i < D / 32; i++)
#pragma unroll
      for (int v = 0; v < 16; v++) red[(qsub * (D / 2) + i * 16 + v) * 64 + lane] = o[i][v];
    if (lg == 0) { red_ml[(qsub * 2 + 0) * 32 + lr] = m; red_ml[(qsub * 2 + 1) * 32 + lr] = l; }
  }
  __syncthreads();
  if (half == 0) {
    const float m_b = red_ml[(qsub * 2 + 0) * 32 + lr], l_b = red_ml[(qsub * 2 + 1) * 32 + lr];
    const float M = fmaxf(m, m_b);
    const float m_ref = M == -INFINITY ? 0.f : M;
    const float ea = __builtin_amdgcn_exp2f(m - m_ref), eb = __builtin_amdgcn_exp2f(m_b - m_ref);
    l = l * ea + l_b * eb;
    if (qg < seq) {
      const size_t piece = (((size_t)b * n + head) * nqb + qb) * max_chunks + chunk;
      float *po = part + piece * G::piece_floats;
      const int qloc = qsub * 32 + lr;
#pragma unroll
      for (int i = 0; i < D / 32; i++)
#pragma unroll
        for (int j = 0; j < 4; j++) {
          f32x4_t w;
#pragma unroll
          for (int r = 0; r < 4; r++) {
            const int v = 4 * j + r;
            w[r] = o[i][v] * ea + red[(qsub * (D / 2) + i * 16 + v) * 64 + lane] * eb;
          }
          *reinterpret_cast<f32x4_t *>(po + (size_t)qloc * D + 32 * i + 8 * j + 4 * lg) = w;
        }
      if (lg == 0) { po[QB * D + qloc] = M; po[QB * D + QB + qloc] = l; }
    }
  }
}

// out[q, :] = sum_c O_c e^{m_c - M} / sum_c l_c e^{m_c - M}; lse = (M + log2 L) ln 2.  One wave per (token, head).
template <int D>
__global__ __launch_bounds__(256) void attn_fwd_combine_kernel(const float *__restrict__ part, bf16_t *__restrict__ out,
                                                               float *__restrict__ lse, int seq, int n, int mbsz, int causal,
                                                               int max_chunks) {
  using G = AttnGeom<D>;
  const int lane = threadIdx.x & 63;
  const size_t w = blockIdx.x * (size_t)4 + (threadIdx.x >> 6);
  if (w >= (size_t)mbsz * n * seq) return;
  const int q = w % seq, head = (w / seq) % n, b = w / ((size_t)seq * n);
  const int nqb = (seq + QB - 1) / QB, qb = q / QB, qloc = q % QB;
  const int nch = (attn_steps(qb, seq, causal) + CH2 - 1) / CH2;
  const float *p0 = part + ((((size_t)b * n + head) * nqb + qb) * max_chunks) * G::piece_floats;
  float M = -INFINITY;
  for (int c = 0; c < nch; c++) M = fmaxf(M, p0[(size_t)c * G::piece_floats + QB * D + qloc]);
  float L = 0.f, acc0 = 0.f, acc1 = 0.f;
  for (int c = 0; c < nch; c++) {
    const float *pc = p0 + (size_t)c * G::piece_floats;
    const float e = __builtin_amdgcn_exp2f(pc[QB * D + qloc] - M);
    L += pc[QB * D + QB + qloc] * e;
    if (D == 128) {
      const float2 v = *reinterpret_cast<const float2 *>(pc + (size_t)qloc * D + 2 * lane);
      acc0 += v.x * e; acc1 += v.y * e;
    } else {
      acc0 += pc[(size_t)qloc * D + lane] * e;
    }
  }
  const float inv = 1.0f / L;
  bf16_t *op = out + ((size_t)b * seq + q) * (n * D) + head * D;
  if (D == 128) {
    typedef bf16_t bf16x2_t __attribute__((ext_vector_type(2)));
    bf16x2_t o2;
    o2[0] = (bf16_t)(acc0 * inv); o2[1] = (bf16_t)(acc1 * inv);
    *reinterpret_cast<bf16x2_t *>(op + 2 * lane) = o2;
  } else {
    op[lane] = (bf16_t)(acc0 * inv);
  }
  if (lane == 0) lse[((size_t)b * n + head) * seq + q] = (M + log2f(L)) * LN2;
}

template <int D>
int launch_fwd(stp_ctx *ctx, const stp_layer_desc *d, const void *qkv, void *out, float *lse, float *ws, size_t ws_bytes,
               hipStream_t s) {
  using G = AttnGeom<D>;
  constexpr size_t smem = (size_t)2 * (G::k_elems + G::v_elems) * sizeof(bf16_t);
  static_assert(smem >= (size_t)(4 * (D / 2) * 64 + 4 * 2 * 32) * sizeof(float), "merge area fits");
  static_assert(smem <= 160 * 1024, "LDS budget");
  auto kern = attn_fwd_bf16_kernel<D>;
  static bool attr_set = false;
  if (!attr_set) {
    STP_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
    attr_set = true;
  }
  const int nqb = (d->seq + QB - 1) / QB;
  const int max_chunks = (attn_steps(nqb - 1, d->seq, d->causal) + CH2 - 1) / CH2;
  const size_t need = (size_t)d->mbsz * d->heads_local * nqb * max_chunks * G::piece_floats * sizeof(float);
  if (!ws || ws_bytes < need)
    return stp_fail(ctx, STP_ENOSPACE, "attention forward: workspace lane too small%s (need %ld bytes)", "", (long)need);
  dim3 grid(nqb, max_chunks, d->heads_local * d->mbsz), block(512);
  float scale_log2 = 1.4426950408889634f / sqrtf((float)D);
  hipLaunchKernelGGL(kern, grid, block, smem, s, (const bf16_t *)qkv, ws, d->seq, d->heads_local, d->causal, max_chunks, scale_log2);
  STP_LAUNCH_CHECK(ctx);
  size_t waves = (size_t)d->mbsz * d->heads_local * d->seq;
  hipLaunchKernelGGL(attn_fwd_combine_kernel<D>, dim3((waves + 3) / 4), dim3(256), 0, s, ws, (bf16_t *)out, lse, d->seq,
                     d->heads_local, d->mbsz, d->causal, max_chunks);
  STP_LAUNCH_CHECK(ctx);
  return STP_OK;
}

}  // namespace

size_t stp_attn_fwd_ws_bytes(const stp_layer_desc *d) {
  const int nqb = (d->seq + QB - 1) / QB;
  const int max_chunks = (attn_steps(nqb - 1, d->seq, d->causal) + CH2 - 1) / CH2;
  return (size_t)d->mbsz * d->heads_local * nqb * max_chunks * (QB * d->head_dim + 2 * QB) * sizeof(float);
}

int stp_launch_attn_fwd_bf16(stp_ctx *ctx, const stp_layer_desc *d, const void *qkv, void *out, float *lse, float *ws,
                             size_t ws_bytes, hipStream_t s) {
  if (d->head_dim == 128) return launch_fwd<128>(ctx, d, qkv, out, lse, ws, ws_bytes, s);
  if (d->head_dim == 64) return launch_fwd<64>(ctx, d, qkv, out, lse, ws, ws_bytes, s);
  return stp_fail(ctx, STP_ESHAPE, "bf16 attention needs head_dim 64 or 128%s");
}

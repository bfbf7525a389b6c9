// Tiled attention forward for bf16 on the CDNA4 matrix cores ("Attention(.)" of Eq. 1:
// the attention core of one TP rank, no communication).
//
// One workgroup = 4 waves handles 128 query rows of one (sequence, head); each wave
// owns 32 query rows and walks the key/value sequence in blocks of 64.  The kernel
// works on the TRANSPOSED score tile, S^T = K Q^T: with the 32x32x16 MFMA the
// accumulator of lane l then holds column q = l % 32, i.e. every softmax statistic
// (running max, running sum, rescale factor) is a per-lane scalar and a row
// reduction is an in-lane loop plus one cross-half shuffle.  The probabilities are
// already in the register layout the next MFMA wants for its B operand
// (O^T += V^T P^T), so P never touches LDS.  V^T fragments come from the V tile as
// it lies in memory ([kv][d]) through the transposing LDS read.
//   K tile  : LDS [64][D + 8]   16-byte fragment reads
//   V tile  : LDS [64][D + 32]  ds_read_b64_tr_b16 fragment reads
// Both are double-buffered through registers (next block's loads in flight during
// the MFMAs of the current one).  Causal: key blocks above the diagonal are never
// visited; the heaviest query blocks are scheduled first.
#include "common.h"

namespace {

constexpr int QB = 128;  // query rows per workgroup
constexpr int KB = 64;   // keys per step

typedef s16x4_t __attribute__((address_space(3))) * lds_s16x4_ptr;

template <int D> struct AttnGeom {
  static constexpr int kp = D + 8;    // K tile pitch (elements)
  static constexpr int vp = D + 32;   // V tile pitch
  static constexpr int k_elems = KB * kp;
  static constexpr int v_elems = KB * vp;
  static constexpr int nld = KB * D / 8 / 256;  // 16-byte chunks per thread per tile
};

template <int D>
__device__ __forceinline__ void kv_load(uint4 (&rk)[AttnGeom<D>::nld], uint4 (&rv)[AttnGeom<D>::nld],
                                        const bf16_t *__restrict__ kbase, size_t ld, int kv0, int seq, int tid) {
#pragma unroll
  for (int i = 0; i < AttnGeom<D>::nld; i++) {
    int q = tid + 256 * i;
    int r = q / (D / 8), c = (q % (D / 8)) * 8;
    bool ok = kv0 + r < seq;
    const bf16_t *p = kbase + (size_t)(kv0 + r) * ld + c;
    rk[i] = ok ? *reinterpret_cast<const uint4 *>(p) : make_uint4(0, 0, 0, 0);
    rv[i] = ok ? *reinterpret_cast<const uint4 *>(p + ld / 3) : make_uint4(0, 0, 0, 0);
  }
}
template <int D>
__device__ __forceinline__ void kv_store(const uint4 (&rk)[AttnGeom<D>::nld], const uint4 (&rv)[AttnGeom<D>::nld],
                                         bf16_t *ks, bf16_t *vs, int tid) {
#pragma unroll
  for (int i = 0; i < AttnGeom<D>::nld; i++) {
    int q = tid + 256 * i;
    int r = q / (D / 8), c = (q % (D / 8)) * 8;
    *reinterpret_cast<uint4 *>(ks + r * AttnGeom<D>::kp + c) = rk[i];
    *reinterpret_cast<uint4 *>(vs + r * AttnGeom<D>::vp + c) = rv[i];
  }
}

template <int D>
__global__ __launch_bounds__(256, 2) void attn_fwd_bf16_kernel(const bf16_t *__restrict__ qkv, bf16_t *__restrict__ out,
                                                               float *__restrict__ lse, int seq, int n, int causal,
                                                               float scale_log2) {
  using G = AttnGeom<D>;
  extern __shared__ __attribute__((aligned(16))) char smem_raw[];
  // stage s: K tile at s*STAGE, V tile at s*STAGE + k_elems (offsets from the LDS base, no pointer tables)
  constexpr int STAGE = G::k_elems + G::v_elems;
  bf16_t *const sbase = reinterpret_cast<bf16_t *>(smem_raw);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lr = lane & 31, lg = lane >> 5;
  const int nqb = (seq + QB - 1) / QB;
  const int qb = nqb - 1 - blockIdx.x;  // heavy (late) query blocks first
  const int head = blockIdx.y, b = blockIdx.z;
  const int a = n * D;
  const size_t ld = 3 * (size_t)a;
  const bf16_t *base = qkv + (size_t)b * seq * ld + head * D;  // Q of this head; K at +a, V at +2a
  const int q_wave0 = qb * QB + wave * 32;
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

  const int q_blk_end = min(seq, qb * QB + QB);              // exclusive
  const int kv_end = causal ? q_blk_end : seq;               // keys this workgroup needs
  const int nkb = (kv_end + KB - 1) / KB;
  const bf16_t *kbase = base + a;

  uint4 rk[G::nld], rv[G::nld];
  kv_load<D>(rk, rv, kbase, ld, 0, seq, tid);
  kv_store<D>(rk, rv, sbase, sbase + G::k_elems, tid);
  __syncthreads();

  for (int kb = 0; kb < nkb; kb++) {
    const int cur = kb & 1;
    const bf16_t *ks_cur = sbase + cur * STAGE, *vs_cur = ks_cur + G::k_elems;
    const int kv0 = kb * KB;
    if (kb + 1 < nkb) kv_load<D>(rk, rv, kbase, ld, kv0 + KB, seq, tid);

    // wave-uniform skip: this wave's 32 queries all precede the key block
    const bool active = !causal || kv0 <= q_wave0 + 31;
    if (active) {
      // ---- S^T[kv, q] = K Q^T
      f32x16_t st[2];
#pragma unroll
      for (int jb = 0; jb < 2; jb++) {
#pragma unroll
        for (int v = 0; v < 16; v++) st[jb][v] = 0.f;
#pragma unroll
        for (int s = 0; s < D / 16; s++) {
          bf16x8_t kf = *reinterpret_cast<const bf16x8_t *>(ks_cur + (32 * jb + lr) * G::kp + 16 * s + 8 * lg);
          st[jb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[s], st[jb], 0, 0, 0);
        }
      }
      // ---- online softmax in the log2 domain; accumulator v of lane l is key
      //      kv0 + 32*jb + 8*(v/4) + 4*(l/32) + v%4, query l%32
      const bool need_mask = (causal && kv0 + KB - 1 > q_wave0) || (kv0 + KB > seq);
      float mx = -INFINITY;
#pragma unroll
      for (int jb = 0; jb < 2; jb++)
#pragma unroll
        for (int v = 0; v < 16; v++) {
          float x = st[jb][v] * scale_log2;
          if (need_mask) {
            int kv = kv0 + 32 * jb + 8 * (v >> 2) + 4 * lg + (v & 3);
            if ((causal && kv > qg) || kv >= seq) x = -INFINITY;
          }
          st[jb][v] = x;
          mx = fmaxf(mx, x);
        }
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      const float m_new = fmaxf(m, mx);
      const float corr = __builtin_amdgcn_exp2f(m - m_new);
      float rs = 0.f;
#pragma unroll
      for (int jb = 0; jb < 2; jb++)
#pragma unroll
        for (int v = 0; v < 16; v++) {
          float p = __builtin_amdgcn_exp2f(st[jb][v] - m_new);
          st[jb][v] = p;
          rs += p;
        }
      rs += __shfl_xor(rs, 32, 64);
      l = l * corr + rs;
      m = m_new;
#pragma unroll
      for (int i = 0; i < D / 32; i++)
#pragma unroll
        for (int v = 0; v < 16; v++) o[i][v] *= corr;

      // ---- O^T[d, q] += V^T P^T ; k-slot i of lane-half g in step (jb, t) is key 32*jb + 16*t + 8*(i/4) + 4*g + i%4
#pragma unroll
      for (int jb = 0; jb < 2; jb++)
#pragma unroll
        for (int t = 0; t < 2; t++) {
          bf16x8_t pf;
#pragma unroll
          for (int i = 0; i < 8; i++) pf[i] = (bf16_t)st[jb][8 * t + i];
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
    }
    if (kb + 1 < nkb) kv_store<D>(rk, rv, sbase + (cur ^ 1) * STAGE, sbase + (cur ^ 1) * STAGE + G::k_elems, tid);
    __syncthreads();
  }

  if (qg < seq) {
    const float inv = 1.0f / l;
    bf16_t *op = out + ((size_t)b * seq + qg) * a + head * D;
#pragma unroll
    for (int db = 0; db < D / 32; db++)
#pragma unroll
      for (int j = 0; j < 4; j++) {
        bf16x4_t w;
#pragma unroll
        for (int r = 0; r < 4; r++) w[r] = (bf16_t)(o[db][4 * j + r] * inv);
        *reinterpret_cast<bf16x4_t *>(op + 32 * db + 8 * j + 4 * lg) = w;
      }
    if (lg == 0) lse[((size_t)b * n + head) * seq + qg] = (m + log2f(l)) * 0.69314718055994531f;
  }
}

template <int D>
int launch_fwd(stp_ctx *ctx, const stp_layer_desc *d, const void *qkv, void *out, float *lse, hipStream_t s) {
  using G = AttnGeom<D>;
  constexpr size_t smem = (size_t)2 * (G::k_elems + G::v_elems) * sizeof(bf16_t);
  auto kern = attn_fwd_bf16_kernel<D>;
  static bool attr_set = false;
  if (!attr_set) {
    STP_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
    attr_set = true;
  }
  dim3 grid((d->seq + QB - 1) / QB, d->heads_local, d->mbsz), block(256);
  float scale_log2 = 1.4426950408889634f / sqrtf((float)D);
  hipLaunchKernelGGL(kern, grid, block, smem, s, (const bf16_t *)qkv, (bf16_t *)out, lse, d->seq, d->heads_local, d->causal, scale_log2);
  STP_LAUNCH_CHECK(ctx);
  return STP_OK;
}

}  // namespace

int stp_launch_attn_fwd_bf16(stp_ctx *ctx, const stp_layer_desc *d, const void *qkv, void *out, float *lse, hipStream_t s) {
  if (d->head_dim == 128) return launch_fwd<128>(ctx, d, qkv, out, lse, s);
  if (d->head_dim == 64) return launch_fwd<64>(ctx, d, qkv, out, lse, s);
  return stp_fail(ctx, STP_ESHAPE, "bf16 attention needs head_dim 64 or 128%s");
}

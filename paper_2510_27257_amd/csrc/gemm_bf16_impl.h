// (included by the four per-layout translation units gemm_bf16_*.hip)
// bf16 GEMM on the CDNA4 matrix cores: C[M,N] = op(A) op(B), fp32 accumulate.
//
// Serves every dense contraction of the units (QKV, out-proj, FC1, FC2 in F; their
// transposed-weight forms in B; the token-contracting forms in W).
//
// Design (gfx950):
//   * one workgroup = 4 waves (2 x 2), block tile BM x BN x 64, each wave owns a
//     (BM/2) x (BN/2) sub-tile as a grid of 32x32 accumulators fed by
//     v_mfma_f32_32x32x16_bf16;
//   * global -> registers -> LDS with two LDS stages: the loads of K-tile kt+1 are in
//     flight while the MFMAs of K-tile kt run, one barrier per K-tile;
//   * an operand whose contraction index is contiguous in memory sits in LDS as
//     [row][64 + 8] and is fetched with one 16-byte LDS read per fragment; an operand
//     whose contraction index is the OUTER index (B = W[in,out] in forward, both
//     operands of the weight-gradient GEMMs) is copied to LDS as it lies in memory,
//     [k][rows + 32], and fetched with the transposing LDS read (ds_read_b64_tr_b16):
//     a 16-lane group reads a 4(k) x 16(row) patch and every lane receives the four
//     k-consecutive values of its own row.  No register or memory transposes.
//   * LDS row pitches (144 B and rows*2+64 B) keep both fetch patterns bank-conflict free;
//   * the blockIdx -> tile map gives each XCD (blockIdx % 8) a contiguous band of tiles
//     walked in groups along M, so tiles resident on one XCD share their A / B panels
//     in that XCD's L2.
#pragma once
#include "common.h"

namespace {

constexpr int BK = 64;
constexpr int KPAD = 8;    // elements; pitch of a k-contiguous tile row = 72 el = 144 B
constexpr int XPAD = 32;   // elements; pitch of a row-contiguous tile = rows + 32

template <int ROWS, bool KC> struct TileGeom {
  static constexpr int pitch = KC ? (BK + KPAD) : (ROWS + XPAD);
  static constexpr int elems = KC ? ROWS * pitch : BK * pitch;
  static constexpr int chunks = ROWS * BK / 8;          // 16-byte chunks per tile
  static constexpr int per_thread = chunks / 256;
};

// Loads this thread's share of a ROWS x 64 operand tile from global memory into registers.
// KC: memory is [row][k] (ld = row pitch);  !KC: memory is [k][row].  Out-of-range chunks are
// read from the (always valid) first element; bit i of the returned mask says chunk i is real.
// The zero-fill happens when the registers are written to LDS, after the MFMAs of the current
// tile, so that all loads stay in flight together (no wait between them).
template <int ROWS, bool KC, int NREG>
__device__ __forceinline__ unsigned tile_load(uint4 (&reg)[NREG], const bf16_t *__restrict__ base,
                                              int ld, int row0, int row_lim, int k0, int k_lim, int tid) {
  static_assert(NREG == TileGeom<ROWS, KC>::per_thread, "register tile size");
  unsigned mask = 0;
#pragma unroll
  for (int i = 0; i < NREG; i++) {
    int q = tid + 256 * i;
    int r, k;
    if (KC) { r = q >> 3; k = (q & 7) * 8; }
    else { k = q / (ROWS / 8); r = (q % (ROWS / 8)) * 8; }
    const bool ok = (row0 + r < row_lim) && (k0 + k < k_lim);
    size_t off = KC ? (size_t)(row0 + r) * ld + (k0 + k) : (size_t)(k0 + k) * ld + (row0 + r);
    off = ok ? off : 0;
    mask |= ok ? (1u << i) : 0u;
    reg[i] = *reinterpret_cast<const uint4 *>(base + off);
  }
  return mask;
}

template <int ROWS, bool KC, int NREG>
__device__ __forceinline__ void tile_store(const uint4 (&reg)[NREG], unsigned mask, bf16_t *lds, int tid) {
  constexpr int P = TileGeom<ROWS, KC>::pitch;
#pragma unroll
  for (int i = 0; i < NREG; i++) {
    int q = tid + 256 * i;
    int r, k;
    if (KC) { r = q >> 3; k = (q & 7) * 8; }
    else { k = q / (ROWS / 8); r = (q % (ROWS / 8)) * 8; }
    bf16_t *p = KC ? lds + r * P + k : lds + k * P + r;
    const bool ok = (mask >> i) & 1u;
    uint4 v;
    v.x = ok ? reg[i].x : 0u; v.y = ok ? reg[i].y : 0u; v.z = ok ? reg[i].z : 0u; v.w = ok ? reg[i].w : 0u;
    *reinterpret_cast<uint4 *>(p) = v;
  }
}

// MFMA operand fragment for the 32 rows starting at `row` and the 16 k-values starting at kk:
// lane l supplies row (l % 32), k = kk + 8*(l/32) .. +7.
template <int ROWS, bool KC>
__device__ __forceinline__ bf16x8_t frag_load(const bf16_t *lds, int row, int kk, int lane) {
  constexpr int P = TileGeom<ROWS, KC>::pitch;
  if (KC) {
    return *reinterpret_cast<const bf16x8_t *>(lds + (row + (lane & 31)) * P + kk + 8 * (lane >> 5));
  } else {
    // transposing read: the 16 lanes of a group point at rows k..k+3 (4 lanes each, 4 columns per lane)
    int k = kk + 8 * (lane >> 5) + ((lane & 15) >> 2);
    int c = row + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
    const bf16_t *p = lds + k * P + c;
    typedef s16x4_t __attribute__((address_space(3))) * lds_ptr_t;
    s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(p));
    s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(p + 4 * P));
    s16x8_t v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8_t, v);
  }
}

struct Epi {
  void *C; int ldc; int c_f32_accum;
  const bf16_t *bias; float bias_scale;
  const bf16_t *resid; int ldr; float resid_scale;
  int mode; bf16_t *C2; const bf16_t *aux; int ld2;
};

enum { EPI_STORE = 0, EPI_GELU_DUAL = 1, EPI_GELU_BWD = 2, EPI_F32_ACCUM = 3 };

template <int BM, int BN, bool A_KC, bool B_KC, int EPI>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(const bf16_t *__restrict__ A, int lda, const bf16_t *__restrict__ B,
                                                        int ldb, int M, int N, int K, int tiles_m, int tiles_n, Epi ep) {
  constexpr int WM = BM / 2, WN = BN / 2, MI = WM / 32, NI = WN / 32;
  using GA = TileGeom<BM, A_KC>;
  using GB = TileGeom<BN, B_KC>;
  extern __shared__ __attribute__((aligned(16))) char smem_raw[];
  // stage s of A at s*STAGE, of B at s*STAGE + GA::elems (plain offsets from the LDS base keep the
  // accesses in the LDS address space; pointer tables would decay to flat addressing)
  constexpr int STAGE = GA::elems + GB::elems;
  bf16_t *const sbase = reinterpret_cast<bf16_t *>(smem_raw);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;

  // ---- XCD-aware tile map: XCD x (= blockIdx % 8) walks the contiguous band [x*per, (x+1)*per)
  const int total = tiles_m * tiles_n;
  int pid = blockIdx.x;
  {
    const int base = total >> 3, rem = total & 7;
    const int x = pid & 7, j = pid >> 3;
    pid = x * base + min(x, rem) + j;
  }
  constexpr int GROUP_M = 4;
  int group = pid / (GROUP_M * tiles_n);
  int first_m = group * GROUP_M;
  int gsize = min(tiles_m - first_m, GROUP_M);
  int tm = first_m + (pid % (GROUP_M * tiles_n)) % gsize;
  int tn = (pid % (GROUP_M * tiles_n)) / gsize;
  const int m0 = tm * BM, n0 = tn * BN;

  f32x16_t acc[MI][NI];
#pragma unroll
  for (int i = 0; i < MI; i++)
#pragma unroll
    for (int j = 0; j < NI; j++)
#pragma unroll
      for (int v = 0; v < 16; v++) acc[i][j][v] = 0.f;

  uint4 ra[GA::per_thread], rb[GB::per_thread];
  const int KT = (K + BK - 1) / BK;
  unsigned ma = tile_load<BM, A_KC>(ra, A, lda, m0, M, 0, K, tid);
  unsigned mb = tile_load<BN, B_KC>(rb, B, ldb, n0, N, 0, K, tid);
  tile_store<BM, A_KC>(ra, ma, sbase, tid);
  tile_store<BN, B_KC>(rb, mb, sbase + GA::elems, tid);
  __syncthreads();

  for (int kt = 0; kt < KT; kt++) {
    const int cur = kt & 1;
    if (kt + 1 < KT) {
      ma = tile_load<BM, A_KC>(ra, A, lda, m0, M, (kt + 1) * BK, K, tid);
      mb = tile_load<BN, B_KC>(rb, B, ldb, n0, N, (kt + 1) * BK, K, tid);
    }
    const bf16_t *a_s = sbase + cur * STAGE, *b_s = sbase + cur * STAGE + GA::elems;
#pragma unroll
    for (int kk = 0; kk < BK; kk += 16) {
      bf16x8_t fa[MI], fb[NI];
#pragma unroll
      for (int i = 0; i < MI; i++) fa[i] = frag_load<BM, A_KC>(a_s, wm * WM + i * 32, kk, lane);
#pragma unroll
      for (int j = 0; j < NI; j++) fb[j] = frag_load<BN, B_KC>(b_s, wn * WN + j * 32, kk, lane);
#pragma unroll
      for (int i = 0; i < MI; i++)
#pragma unroll
        for (int j = 0; j < NI; j++)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < KT) {
      tile_store<BM, A_KC>(ra, ma, sbase + (cur ^ 1) * STAGE, tid);
      tile_store<BN, B_KC>(rb, mb, sbase + (cur ^ 1) * STAGE + GA::elems, tid);
    }
    __syncthreads();
  }

  // ---- epilogue.  Accumulator v of lane l is C[32*i + 8*(v/4) + 4*(l/32) + v%4][32*j + l%32].
  // Each wave stages one 32 x WN strip at a time in its own LDS area (fp32, pitch WN + 8 keeps the two
  // lane halves on different banks) and reads it back row-wise, 8 consecutive columns per lane, so
  // that every global access of the epilogue (C, C2, residual, aux, bias) is a 16- or 32-byte vector.
  constexpr int SP = WN + 8;
  static_assert((size_t)4 * 32 * SP * sizeof(float) <= (size_t)2 * (GA::elems + GB::elems) * sizeof(bf16_t), "staging fits");
  float *stage = reinterpret_cast<float *>(smem_raw) + wave * (32 * SP);
  const int lr = lane & 31, lg = lane >> 5;
  const bool has_bias = ep.bias != nullptr, has_resid = ep.resid != nullptr;
  constexpr int LPR = WN / 8;             // lanes per staged row
  constexpr int PASSES = 32 * LPR / 64;
#pragma unroll
  for (int i = 0; i < MI; i++) {
#pragma unroll
    for (int j = 0; j < NI; j++)
#pragma unroll
      for (int v = 0; v < 16; v++) stage[(8 * (v >> 2) + 4 * lg + (v & 3)) * SP + 32 * j + lr] = acc[i][j][v];
    __syncthreads();
#pragma unroll 1
    for (int p = 0; p < PASSES; p++) {
      const int idx = p * 64 + lane;
      const int r = idx / LPR, c = (idx % LPR) * 8;
      const int row = m0 + wm * WM + i * 32 + r, col = n0 + wn * WN + c;
      if (row < M && col < N) {
        float val[8];
        Vec8<float>::load(stage + r * SP + c, val);
        if (has_bias) {
          float b[8];
          Vec8<bf16_t>::load(ep.bias + col, b);
#pragma unroll
          for (int e = 0; e < 8; e++) val[e] += b[e] * ep.bias_scale;
        }
        if (has_resid) {
          float rr[8];
          Vec8<bf16_t>::load(ep.resid + (size_t)row * ep.ldr + col, rr);
#pragma unroll
          for (int e = 0; e < 8; e++) val[e] += rr[e] * ep.resid_scale;
        }
        if (EPI == EPI_F32_ACCUM) {
          float *cp = reinterpret_cast<float *>(ep.C) + (size_t)row * ep.ldc + col;
          float old[8];
          Vec8<float>::load(cp, old);
#pragma unroll
          for (int e = 0; e < 8; e++) old[e] += val[e];
          Vec8<float>::store(cp, old);
        } else {
          if (EPI == EPI_GELU_BWD) {
            float h[8];
            Vec8<bf16_t>::load(ep.aux + (size_t)row * ep.ld2 + col, h);
#pragma unroll
            for (int e = 0; e < 8; e++) val[e] *= gelu_grad_f(h[e]);
          }
          bf16x8_t o;
#pragma unroll
          for (int e = 0; e < 8; e++) o[e] = (bf16_t)val[e];
          *reinterpret_cast<bf16x8_t *>(reinterpret_cast<bf16_t *>(ep.C) + (size_t)row * ep.ldc + col) = o;
          if (EPI == EPI_GELU_DUAL) {
            float gv[8];
#pragma unroll
            for (int e = 0; e < 8; e++) gv[e] = gelu_f((float)o[e]);
            Vec8<bf16_t>::store(ep.C2 + (size_t)row * ep.ld2 + col, gv);
          }
        }
      }
    }
    __syncthreads();
  }
}

template <int BM, int BN, bool A_KC, bool B_KC, int EPI>
int launch_cfg(stp_ctx *ctx, const stp_gemm_args *a, const Epi &ep, hipStream_t s) {
  using GA = TileGeom<BM, A_KC>;
  using GB = TileGeom<BN, B_KC>;
  constexpr size_t smem = (size_t)2 * (GA::elems + GB::elems) * sizeof(bf16_t);
  static_assert(smem <= 160 * 1024, "LDS budget");
  auto kern = gemm_bf16_kernel<BM, BN, A_KC, B_KC, EPI>;
  static bool attr_set = false;   // the attribute is per function; setting it twice is harmless
  if (!attr_set) {
    STP_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
    attr_set = true;
  }
  int tiles_m = (a->M + BM - 1) / BM, tiles_n = (a->N + BN - 1) / BN;
  hipLaunchKernelGGL(kern, dim3(tiles_m * tiles_n), dim3(256), smem, s, (const bf16_t *)a->A, a->lda, (const bf16_t *)a->B,
                     a->ldb, a->M, a->N, a->K, tiles_m, tiles_n, ep);
  STP_LAUNCH_CHECK(ctx);
  return STP_OK;
}

template <bool A_KC, bool B_KC, int EPI>
int launch_tile(stp_ctx *ctx, const stp_gemm_args *a, const Epi &ep, hipStream_t s) {
  long t256 = (long)((a->M + 255) / 256) * ((a->N + 255) / 256);
  if (t256 >= 96) return launch_cfg<256, 256, A_KC, B_KC, EPI>(ctx, a, ep, s);
  return launch_cfg<128, 128, A_KC, B_KC, EPI>(ctx, a, ep, s);
}

template <bool A_KC, bool B_KC>
int launch_layout(stp_ctx *ctx, const stp_gemm_args *a, hipStream_t s) {
  Epi ep;
  ep.C = a->C; ep.ldc = a->ldc; ep.c_f32_accum = a->c_f32_accum;
  ep.bias = (const bf16_t *)a->bias; ep.bias_scale = a->bias_scale;
  ep.resid = (const bf16_t *)a->resid; ep.ldr = a->ldr; ep.resid_scale = a->resid_scale;
  ep.mode = a->epilogue; ep.C2 = (bf16_t *)a->C2; ep.aux = (const bf16_t *)a->aux; ep.ld2 = a->ld2;
  if (a->c_f32_accum) return launch_tile<A_KC, B_KC, EPI_F32_ACCUM>(ctx, a, ep, s);
  if (a->epilogue == 1) return launch_tile<A_KC, B_KC, EPI_GELU_DUAL>(ctx, a, ep, s);
  if (a->epilogue == 2) return launch_tile<A_KC, B_KC, EPI_GELU_BWD>(ctx, a, ep, s);
  return launch_tile<A_KC, B_KC, EPI_STORE>(ctx, a, ep, s);
}

}  // namespace

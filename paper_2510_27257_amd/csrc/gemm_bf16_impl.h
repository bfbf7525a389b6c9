// (included by the four per-layout translation units gemm_bf16_*.hip)
// bf16 GEMM on the CDNA4 matrix cores: C[M,N] = op(A) op(B), fp32 accumulate.
//
// Serves every dense contraction of the units (QKV, out-proj, FC1, FC2 in F; their
// transposed-weight forms in B; the token-contracting forms in W).
//
// Two kernels share the fragment scheme, the tile map and the epilogue:
//   * gemm_bf16_dma_kernel (further down): direct-to-LDS loads, 4-stage ring of 32-deep K-tiles, the path of
//     every problem with K a multiple of 32;
//   * gemm_bf16_kernel: the fallback for any K and for operands of 2 GiB and more, described here.
//
// Fallback design (gfx950):
//   * one workgroup = WAVES_M x WAVES_N waves, block tile BM x BN x 64, each wave owns a
//     (BM/WAVES_M) x (BN/WAVES_N) sub-tile as a grid of 32x32 accumulators fed by v_mfma_f32_32x32x16_bf16;
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
#include "lds_dma.h"
#include <utility>
#include <stdlib.h>

namespace {

constexpr int BK = 64;
constexpr int KPAD = 8;    // elements; pitch of a k-contiguous tile row = 72 el = 144 B
constexpr int XPAD = 32;   // elements; pitch of a row-contiguous tile = rows + 32

template <int ROWS, bool KC> struct TileGeom {
  static constexpr int pitch = KC ? (BK + KPAD) : (ROWS + XPAD);
  static constexpr int elems = KC ? ROWS * pitch : BK * pitch;
  static constexpr int chunks = ROWS * BK / 8;          // 16-byte chunks per tile
};

// Loads this thread's share of a ROWS x 64 operand tile from global memory into registers.
// KC: memory is [row][k] (ld = row pitch);  !KC: memory is [k][row].  Out-of-range chunks are
// read from the (always valid) first element; bit i of the returned mask says chunk i is real.
// The zero-fill happens when the registers are written to LDS, after the MFMAs of the current
// tile, so that all loads stay in flight together (no wait between them).
template <int ROWS, bool KC, int NTH, int NREG>
__device__ __forceinline__ unsigned tile_load(uint4 (&reg)[NREG], const bf16_t *__restrict__ base,
                                              int ld, int row0, int row_lim, int k0, int k_lim, int tid) {
  static_assert(NREG * NTH == TileGeom<ROWS, KC>::chunks, "register tile size");
  unsigned mask = 0;
#pragma unroll
  for (int i = 0; i < NREG; i++) {
    int q = tid + NTH * i;
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

template <int ROWS, bool KC, int NTH, int NREG>
__device__ __forceinline__ void tile_store(const uint4 (&reg)[NREG], unsigned mask, bf16_t *lds, int tid) {
  constexpr int P = TileGeom<ROWS, KC>::pitch;
#pragma unroll
  for (int i = 0; i < NREG; i++) {
    int q = tid + NTH * i;
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
#ifdef STP_GEMM_TRACE
  long long *trace;   // measurement build only: 4 wall-clock stamps per workgroup
#endif
  void *C; int ldc; int c_f32_accum;
  const bf16_t *bias; float bias_scale;
  const bf16_t *resid; int ldr; float resid_scale;
  int mode; bf16_t *C2; const bf16_t *aux; int ld2;
};

enum { EPI_STORE = 0, EPI_GELU_DUAL = 1, EPI_GELU_BWD = 2, EPI_F32_ACCUM = 3 };

// XCD-aware tile map: workgroups are dealt round-robin to the 8 XCDs, so XCD x (= blockIdx % 8) is given
// the contiguous band [x*total/8, (x+1)*total/8) of a tile order that walks groups of 4 tile-rows
// column by column: tiles resident on one XCD share their A / B panels in that XCD's L2.
__device__ __forceinline__ void map_tile(int tiles_m, int tiles_n, int &tm, int &tn) {
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
  tm = first_m + (pid % (GROUP_M * tiles_n)) % gsize;
  tn = (pid % (GROUP_M * tiles_n)) / gsize;
}

// Epilogue.  Accumulator v of lane l is C[32*i + 8*(v/4) + 4*(l/32) + v%4][32*j + l%32].
// Each wave stages one 32 x WN strip at a time in its own LDS area (fp32, pitch WN + 8 keeps the two
// lane halves on different banks) and reads it back row-wise, 8 consecutive columns per lane, so
// that every global access of the epilogue (C, C2, residual, aux, bias) is a 16- or 32-byte vector.
// The staging area is private to the wave (LDS operations of a wave complete in order), so no barrier
// is needed.  What the epilogue reads from global memory (residual, aux, the fp32 accumulator) is
// fetched one strip ahead, all passes of a strip at once, so that its latency is paid once per tile
// and not once per pass.  Rows / columns past M / N are read from a clamped address and never stored.
// The caller guarantees that the operand stages in LDS are dead (barrier after the last K-tile).
template <int MI, int NI, int WN, int EPI>
__device__ __forceinline__ void store_tile(f32x16_t (&acc)[MI][NI], float *stage, int row_base, int col_base, int M, int N,
                                           const Epi &ep, int lane) {
  constexpr int SP = WN + 8;
  const int lr = lane & 31, lg = lane >> 5;
  const bool has_bias = ep.bias != nullptr, has_resid = ep.resid != nullptr;
  constexpr int LPR = WN / 8;             // lanes per staged row
  constexpr int PASSES = 32 * LPR / 64;
  constexpr bool ACC = EPI == EPI_F32_ACCUM, AUX = EPI == EPI_GELU_BWD;
  // pass p of a strip: staged row r_p, columns c_p .. c_p+7 (the same for every strip)
  int pr[PASSES], pc[PASSES];
  float bias[PASSES][8];
#pragma unroll
  for (int p = 0; p < PASSES; p++) {
    const int idx = p * 64 + lane;
    pr[p] = idx / LPR;
    pc[p] = col_base + (idx % LPR) * 8;
#pragma unroll
    for (int e = 0; e < 8; e++) bias[p][e] = 0.f;
    if (has_bias) {
      Vec8<bf16_t>::load(ep.bias + min(pc[p], N - 8), bias[p]);
#pragma unroll
      for (int e = 0; e < 8; e++) bias[p][e] *= ep.bias_scale;
    }
  }
  // what strip i needs from global memory
  struct Pre { uint4 lo[PASSES], hi[PASSES]; };   // resid / aux: lo (8 bf16); fp32 accumulator: lo, hi (8 floats)
  auto fetch = [&](int i, Pre &f) {
#pragma unroll
    for (int p = 0; p < PASSES; p++) {
      const size_t row = (size_t)min(row_base + i * 32 + pr[p], M - 1);
      const int col = min(pc[p], N - 8);
      if (ACC) {
        const uint4 *cp = reinterpret_cast<const uint4 *>(reinterpret_cast<const float *>(ep.C) + row * ep.ldc + col);
        const uint4 a = cp[0], b = cp[1];
        f.lo[p].x = a.x; f.lo[p].y = a.y; f.lo[p].z = a.z; f.lo[p].w = a.w;
        f.hi[p].x = b.x; f.hi[p].y = b.y; f.hi[p].z = b.z; f.hi[p].w = b.w;
      } else if (AUX) {
        const uint4 a = *reinterpret_cast<const uint4 *>(ep.aux + row * ep.ld2 + col);
        f.lo[p].x = a.x; f.lo[p].y = a.y; f.lo[p].z = a.z; f.lo[p].w = a.w;
      } else if (has_resid) {
        const uint4 a = *reinterpret_cast<const uint4 *>(ep.resid + row * ep.ldr + col);
        f.lo[p].x = a.x; f.lo[p].y = a.y; f.lo[p].z = a.z; f.lo[p].w = a.w;
      }
    }
  };
  auto strip = [&](int i, const Pre &f) {
#pragma unroll
    for (int j = 0; j < NI; j++)
#pragma unroll
      for (int v = 0; v < 16; v++) stage[(8 * (v >> 2) + 4 * lg + (v & 3)) * SP + 32 * j + lr] = acc[i][j][v];
#pragma unroll
    for (int p = 0; p < PASSES; p++) {
      const int row = row_base + i * 32 + pr[p], col = pc[p];
      float val[8];
      Vec8<float>::load(stage + pr[p] * SP + (col - col_base), val);
#pragma unroll
      for (int e = 0; e < 8; e++) val[e] += bias[p][e];
      if (ACC) {
        float old[8];
        old[0] = __builtin_bit_cast(float, f.lo[p].x); old[1] = __builtin_bit_cast(float, f.lo[p].y);
        old[2] = __builtin_bit_cast(float, f.lo[p].z); old[3] = __builtin_bit_cast(float, f.lo[p].w);
        old[4] = __builtin_bit_cast(float, f.hi[p].x); old[5] = __builtin_bit_cast(float, f.hi[p].y);
        old[6] = __builtin_bit_cast(float, f.hi[p].z); old[7] = __builtin_bit_cast(float, f.hi[p].w);
#pragma unroll
        for (int e = 0; e < 8; e++) old[e] += val[e];
        if (row < M && col < N) Vec8<float>::store(reinterpret_cast<float *>(ep.C) + (size_t)row * ep.ldc + col, old);
      } else {
        if (AUX || has_resid) {
          uint4 raw;
          raw.x = f.lo[p].x; raw.y = f.lo[p].y; raw.z = f.lo[p].z; raw.w = f.lo[p].w;
          const bf16x8_t h8 = __builtin_bit_cast(bf16x8_t, raw);
#pragma unroll
          for (int e = 0; e < 8; e++) {
            if (AUX) val[e] *= gelu_grad_t<bf16_t>((float)h8[e]);
            else val[e] += (float)h8[e] * ep.resid_scale;
          }
        }
        bf16x8_t o;
#pragma unroll
        for (int e = 0; e < 8; e++) o[e] = (bf16_t)val[e];
        if (row < M && col < N) {
          *reinterpret_cast<bf16x8_t *>(reinterpret_cast<bf16_t *>(ep.C) + (size_t)row * ep.ldc + col) = o;
          if (EPI == EPI_GELU_DUAL) {
            float gv[8];
#pragma unroll
            for (int e = 0; e < 8; e++) gv[e] = gelu_t<bf16_t>((float)o[e]);
            Vec8<bf16_t>::store(ep.C2 + (size_t)row * ep.ld2 + col, gv);
          }
        }
      }
    }
  };
  // strips alternate between two prefetch buffers; MI is 2 or 4
  Pre f0, f1;
  fetch(0, f0);
#pragma unroll
  for (int i = 0; i < MI; i += 2) {
    if (i + 1 < MI) fetch(i + 1, f1);
    strip(i, f0);
    if (i + 2 < MI) fetch(i + 2, f0);
    if (i + 1 < MI) strip(i + 1, f1);
  }
}

template <int BM, int BN, int WAVES_M, int WAVES_N, bool A_KC, bool B_KC, int EPI>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N) void gemm_bf16_kernel(const bf16_t *__restrict__ A, int lda, const bf16_t *__restrict__ B,
                                                        int ldb, int M, int N, int K, int tiles_m, int tiles_n, Epi ep) {
  constexpr int NTH = 64 * WAVES_M * WAVES_N;
  constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N, MI = WM / 32, NI = WN / 32;
  using GA = TileGeom<BM, A_KC>;
  using GB = TileGeom<BN, B_KC>;
  extern __shared__ __attribute__((aligned(16))) char smem_raw[];
  // stage s of A at s*STAGE, of B at s*STAGE + GA::elems (plain offsets from the LDS base keep the
  // accesses in the LDS address space; pointer tables would decay to flat addressing)
  constexpr int STAGE = GA::elems + GB::elems;
  bf16_t *const sbase = reinterpret_cast<bf16_t *>(smem_raw);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;

  int tm, tn;
  map_tile(tiles_m, tiles_n, tm, tn);
  const int m0 = tm * BM, n0 = tn * BN;

  f32x16_t acc[MI][NI];
#pragma unroll
  for (int i = 0; i < MI; i++)
#pragma unroll
    for (int j = 0; j < NI; j++)
#pragma unroll
      for (int v = 0; v < 16; v++) acc[i][j][v] = 0.f;

  uint4 ra[GA::chunks / NTH], rb[GB::chunks / NTH];
  const int KT = (K + BK - 1) / BK;
  unsigned ma = tile_load<BM, A_KC, NTH>(ra, A, lda, m0, M, 0, K, tid);
  unsigned mb = tile_load<BN, B_KC, NTH>(rb, B, ldb, n0, N, 0, K, tid);
  tile_store<BM, A_KC, NTH>(ra, ma, sbase, tid);
  tile_store<BN, B_KC, NTH>(rb, mb, sbase + GA::elems, tid);
  __syncthreads();

  for (int kt = 0; kt < KT; kt++) {
    const int cur = kt & 1;
    if (kt + 1 < KT) {
      ma = tile_load<BM, A_KC, NTH>(ra, A, lda, m0, M, (kt + 1) * BK, K, tid);
      mb = tile_load<BN, B_KC, NTH>(rb, B, ldb, n0, N, (kt + 1) * BK, K, tid);
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
      tile_store<BM, A_KC, NTH>(ra, ma, sbase + (cur ^ 1) * STAGE, tid);
      tile_store<BN, B_KC, NTH>(rb, mb, sbase + (cur ^ 1) * STAGE + GA::elems, tid);
    }
    __syncthreads();
  }

  store_tile<MI, NI, WN, EPI>(acc, reinterpret_cast<float *>(smem_raw) + wave * (32 * (WN + 8)), m0 + wm * WM, n0 + wn * WN, M, N,
                              ep, lane);
}


// =====================================================================================================
// Kernel with direct-to-LDS loads and a 4-stage pipeline (the path every large GEMM takes).
//
// buffer_load_dwordx4 ... lds moves 16 bytes per lane from global memory straight into LDS (lane i of a
// wave instruction lands at M0 + 16*i): no staging registers, no ds_write, and the loads of three
// K-tiles (32 deep each) stay in flight behind the MFMAs of the current one.  The buffer form (resource
// descriptor in SGPRs, one 32-bit byte offset per lane, the K position in a scalar offset) is used
// because the issue of a load with 64-bit per-lane addresses holds the SIMD's vector register ports
// long enough to stall the MFMAs of the other wave on that SIMD (measured: about 15 % of a K-tile).
// A wave instruction fills 1 KB of LDS contiguously, so padding is impossible; bank conflicts are
// avoided by permuting WHICH global chunk each lane fetches (an XOR swizzle applied on the global
// side and undone in the fragment address):
//   k-contiguous operand : tile [rows][32], 4 chunks per row; chunk c of row r sits in slot c ^ ((r>>2)&3)
//   row-contiguous operand: tile [32][rows], rows/8 chunks per k-row; chunk c of k-row k sits in slot
//                           c ^ (4*(k&3))   (read back with ds_read_b64_tr_b16)
//
// Schedule.  Two waves per SIMD run freely (no phase lock); each wave software-pipelines its fragments:
// the LDS reads of the next 16-deep step are issued before the 8..16 MFMAs of the current one, so LDS
// latency hides behind the wave's own MFMAs and the other wave on the SIMD fills what is left.  All
// fragment reads are inline assembly with explicit lgkmcnt waits: the compiler neither tracks the
// direct-to-LDS loads nor may it order LDS reads behind them (through builtins it would wait for
// vmcnt(0) before every transposing read).  One s_barrier per K-tile, between its two steps:
//     s_waitcnt vmcnt(2 tiles' worth) lgkmcnt(0) ; s_barrier
// after it tile kt+1 has landed for every wave, and no wave has a read of stage kt outstanding (both
// fragment sets of tile kt are in registers), so stage kt is refilled with tile kt+4 right there.
// Rows past M / N are fetched from a clamped (valid) address and never stored; K must be a multiple
// of 32 and each operand must span less than 2 GiB.
// =====================================================================================================
constexpr int DK = 32;         // K-tile depth of the DMA kernel
constexpr int DSTAGES = 4;

template <int ROWS, bool KC, int NWAVES>
struct DmaOp {
  static_assert(ROWS % 16 == 0, "a tile is a whole number of 1 KB pieces per K-tile");
  static_assert(KC || (ROWS / 8) % 16 == 0, "the chunk permutation of a row-contiguous tile works on blocks of 16 chunks");
  static constexpr int PIECES = ROWS / 16;                               // 1 KB pieces (wave instructions) per K-tile
  static constexpr int NINST = (PIECES + NWAVES - 1) / NWAVES;           // issue slots per wave per K-tile
  static constexpr bool EVEN = PIECES % NWAVES == 0;                     // every slot of every wave has a piece
  static constexpr int bytes = ROWS * DK * 2;
  static constexpr int CPR = ROWS / 8;                   // 16-byte chunks per k-row (row-contiguous operand)
  static constexpr int LDS_OPS_PER_FRAG = KC ? 1 : 2;
  // piece that slot j of wave `wave` loads; pieces >= PIECES do not exist (the slot then loads piece 0 again,
  // into a dump area: every wave issues the same number of loads per K-tile, which the vmcnt waits rely on)
  static __device__ __forceinline__ int piece(int j, int wave) { return wave + NWAVES * j; }
  // byte offset (from the operand base, K-tile 0) of the chunk that lane `lane` of this wave's j-th
  // instruction must fetch
  static __device__ __forceinline__ unsigned chunk_offset(int j, int wave, int lane, int ld, int row0, int row_lim) {
    const int pc = piece(j, wave);
    const int p = (pc < PIECES ? pc : 0) * 64 + lane;
    if (KC) {
      const int r = p >> 2, c = (p & 3) ^ ((r >> 2) & 3);
      const int row = min(row0 + r, row_lim - 1);
      return ((unsigned)row * (unsigned)ld + c * 8) * 2u;
    } else {
      const int k = p / CPR, c = (p % CPR) ^ (4 * (k & 3));
      int col = row0 + c * 8;
      col = col < row_lim ? col : 0;
      return ((unsigned)k * (unsigned)ld + col) * 2u;
    }
  }
  // LDS byte offsets (within a tile) from which the fragments of rows row .. row + 32*NF - 1 are read:
  // k-contiguous: one address per 16-deep half (fragment i adds 32 rows = 2048 bytes as an immediate);
  // row-contiguous: one address per fragment (the half adds 16 k-rows as an immediate).
  template <int NF>
  static __device__ __forceinline__ void frag_bases(unsigned (&ad)[KC ? 2 : NF], int row, int lane) {
    if (KC) {
      const int r = row + (lane & 31);
#pragma unroll
      for (int h = 0; h < 2; h++) {
        const int c = 2 * h + (lane >> 5);
        ad[h] = (r * 4 + (c ^ ((r >> 2) & 3))) * 16;
      }
    } else {
      const int k = 8 * (lane >> 5) + ((lane & 15) >> 2);
#pragma unroll
      for (int i = 0; i < NF; i++) {
        const int col = row + 32 * i + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
        ad[i] = (k * CPR + ((col >> 3) ^ (4 * (k & 3)))) * 16 + (col & 7) * 2;
      }
    }
  }
  // issues the reads of the NF fragments of half H (k = 16*H .. 16*H+15) of the tile at LDS address `tile`
  template <int H, int NF, int... I>
  static __device__ __forceinline__ void frag_issue(u32x4_t (&f)[NF], const unsigned (&ad)[KC ? 2 : NF], unsigned tile,
                                                    std::integer_sequence<int, I...>) {
    if constexpr (KC) {
      const unsigned a = ad[H] + tile;
      ((f[I] = lds_read_b128<I * 2048>(a)), ...);
    } else {
      ((f[I] = lds_read_tr16<H * 16 * CPR * 16, 4 * CPR * 16>(ad[I] + tile)), ...);
    }
  }
};

template <int BM, int BN, int WAVES_M, int WAVES_N, int NSTG, bool A_KC, bool B_KC, int EPI>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N) void gemm_bf16_dma_kernel(const bf16_t *__restrict__ A, int lda, int a_bytes,
                                                            const bf16_t *__restrict__ B, int ldb, int b_bytes, int M, int N, int K,
                                                            int tiles_m, int tiles_n, Epi ep) {
  constexpr int NWAVES = WAVES_M * WAVES_N;
  constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N, MI = WM / 32, NI = WN / 32;
  using OA = DmaOp<BM, A_KC, NWAVES>;
  using OB = DmaOp<BN, B_KC, NWAVES>;
  constexpr int STAGE_BYTES = OA::bytes + OB::bytes;
  constexpr int LOADS_PER_TILE = OA::NINST + OB::NINST;
  constexpr int READS_PER_STEP = MI * OA::LDS_OPS_PER_FRAG + NI * OB::LDS_OPS_PER_FRAG;
  // lgkmcnt is a 4-bit counter: with 16 reads per step the wait for "the previous step's reads" also waits for
  // the first read of the step just issued (the reads of a wave complete in order)
  constexpr int READS_WAIT = READS_PER_STEP < 15 ? READS_PER_STEP : 15;
  static_assert(READS_PER_STEP <= 16, "one step's fragment reads must fit the lgkmcnt counter");
  extern __shared__ __attribute__((aligned(1024))) char smem_raw[];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
#ifdef STP_GEMM_TRACE
  const long long tr0 = wall_clock64();
#endif
  const int wave_s = __builtin_amdgcn_readfirstlane(wave);   // same value, known wave-uniform: LDS targets of the loads stay scalar
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;
  int tm, tn;
  map_tile(tiles_m, tiles_n, tm, tn);
  const int m0 = tm * BM, n0 = tn * BN;

  const __amdgpu_buffer_rsrc_t ra = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(A), 0, a_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rb = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(B), 0, b_bytes, 0x00020000);
  unsigned offa[OA::NINST], offb[OB::NINST];
#pragma unroll
  for (int j = 0; j < OA::NINST; j++) offa[j] = OA::chunk_offset(j, wave, lane, lda, m0, M);
#pragma unroll
  for (int j = 0; j < OB::NINST; j++) offb[j] = OB::chunk_offset(j, wave, lane, ldb, n0, N);
  const unsigned stepa = (A_KC ? (unsigned)DK : (unsigned)DK * lda) * 2u;
  const unsigned stepb = (B_KC ? (unsigned)DK : (unsigned)DK * ldb) * 2u;

  unsigned ada[A_KC ? 2 : MI], adb[B_KC ? 2 : NI];
  OA::template frag_bases<MI>(ada, wm * WM, lane);
  OB::template frag_bases<NI>(adb, wn * WN, lane);
  const unsigned lds0 = (unsigned)(size_t)(const __attribute__((address_space(3))) char *)smem_raw;

  f32x16_t acc[MI][NI];
#pragma unroll
  for (int i = 0; i < MI; i++)
#pragma unroll
    for (int j = 0; j < NI; j++)
#pragma unroll
      for (int v = 0; v < 16; v++) acc[i][j][v] = 0.f;

  const int KT = K / DK;
  // The direct-to-LDS loads form one stream, tile after tile, each tile as A's instructions then B's.
  // Issuing a load holds the wave until the address unit takes it, so the loads are placed one at a time
  // between MFMAs (whose execution covers the hold) instead of in a burst behind the barrier, where the
  // eight waves would queue on the address FIFO with the matrix pipes idle.  Per K-tile kt the first
  // LF loads of tile kt+4 go into the MFMA block that follows the barrier (stage kt is free from there on)
  // and the remaining LS loads into the MFMA block before the next barrier.
#define STP_ISSUE(q, ktile, stage)                                                                               \
  do {                                                                                                           \
    const int kt_ = min((ktile), KT - 1);                                                                        \
    char *st_ = smem_raw + (stage) * STAGE_BYTES;                                                                \
    if ((q) < OA::NINST) {                                                                                       \
      const int pc_ = OA::piece((q), wave_s);                                                                    \
      char *dst_ = (OA::EVEN || pc_ < OA::PIECES) ? st_ + pc_ * 1024 : smem_raw + NSTG * STAGE_BYTES;            \
      dma_load16(ra, dst_, offa[(q) < OA::NINST ? (q) : 0], kt_ * stepa);                                        \
    } else {                                                                                                     \
      const int pc_ = OB::piece((q) - OA::NINST, wave_s);                                                        \
      char *dst_ = (OB::EVEN || pc_ < OB::PIECES) ? st_ + OA::bytes + pc_ * 1024 : smem_raw + NSTG * STAGE_BYTES; \
      dma_load16(rb, dst_, offb[(q) >= OA::NINST ? (q) - OA::NINST : 0], kt_ * stepb);                           \
    }                                                                                                            \
  } while (0)
  u32x4_t fa0[MI], fb0[NI], fa1[MI], fb1[NI];
  constexpr int LF = (LOADS_PER_TILE + 1) / 2, LS = LOADS_PER_TILE - LF;
  // prologue: tiles 0 .. NSTG-2 and the first LF loads of tile NSTG-1
#pragma unroll
  for (int t = 0; t < NSTG; t++)
#pragma unroll
    for (int q = 0; q < (t < NSTG - 1 ? LOADS_PER_TILE : LF); q++) STP_ISSUE(q, t, t);

  using SeqM = std::make_integer_sequence<int, MI>;
  using SeqN = std::make_integer_sequence<int, NI>;
#define STP_READ(H, FA, FB, stage)                                                   \
  do {                                                                               \
    const unsigned t_ = lds0 + (unsigned)(stage) * STAGE_BYTES;                      \
    OA::template frag_issue<H>(FA, ada, t_, SeqM{});                                 \
    OB::template frag_issue<H>(FB, adb, t_ + OA::bytes, SeqN{});                     \
    __builtin_amdgcn_sched_barrier(0);                                               \
  } while (0)
  // MI*NI MFMAs with loads Q0 .. Q0+NQ-1 of tile `ktile` spread evenly between them
#define STP_MFMAS(FA, FB, Q0, NQ, ktile, stage)                                      \
  do {                                                                               \
    lds_tie(FA);                                                                     \
    lds_tie(FB);                                                                     \
    _Pragma("unroll") for (int i = 0; i < MI; i++)                                   \
      _Pragma("unroll") for (int j = 0; j < NI; j++) {                               \
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, FA[i]), __builtin_bit_cast(bf16x8_t, FB[j]), \
                                                            acc[i][j], 0, 0, 0);     \
        _Pragma("unroll") for (int r = 0; r < (NQ); r++)                             \
          if (i * NI + j == max(0, ((r + 1) * MI * NI) / ((NQ) + 1) - 1)) {          \
            __builtin_amdgcn_sched_barrier(0);                                       \
            STP_ISSUE((Q0) + r, ktile, stage);                                       \
            __builtin_amdgcn_sched_barrier(0);                                       \
          }                                                                          \
      }                                                                              \
    __builtin_amdgcn_sched_barrier(0);                                               \
  } while (0)

  asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"((NSTG - 2) * LOADS_PER_TILE + LF) : "memory");
#ifdef STP_GEMM_TRACE
  const long long tr1 = wall_clock64();
#endif
  STP_READ(0, fa0, fb0, 0);

  for (int kt = 0; kt < KT; kt++) {
    const int st = kt % NSTG;
    STP_READ(1, fa1, fb1, st);
    lds_wait<READS_WAIT>();              // the reads of half 0 (issued one step ago) have returned
    STP_MFMAS(fa0, fb0, LF, LS, kt + NSTG - 1, (kt + NSTG - 1) % NSTG);
    // tile kt+1 has landed once at most (NSTG-2) tiles' worth of this wave's loads remain in flight;
    // lgkmcnt(0): this wave's reads of stage st are complete, so after the barrier the stage is free
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"((NSTG - 2) * LOADS_PER_TILE) : "memory");
    __builtin_amdgcn_sched_barrier(0);
    STP_READ(0, fa0, fb0, (kt + 1) % NSTG);   // past the last tile this reads a stale stage; never used
    lds_wait<READS_WAIT>();
    STP_MFMAS(fa1, fb1, 0, LF, kt + NSTG, st);
  }
#undef STP_READ
#undef STP_MFMAS
#undef STP_ISSUE
  // drain the (redundant) tail loads and reads before the stages are reused as epilogue staging
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
  lds_tie(fa0);
  lds_tie(fb0);
#ifdef STP_GEMM_TRACE
  const long long tr2 = wall_clock64();
#endif
  store_tile<MI, NI, WN, EPI>(acc, reinterpret_cast<float *>(smem_raw) + wave * (32 * (WN + 8)), m0 + wm * WM, n0 + wn * WN, M, N,
                              ep, lane);
#ifdef STP_GEMM_TRACE
  if (ep.trace) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    const long long tr3 = wall_clock64();
    if (tid == 0) {
      unsigned hw;
      asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(hw));
      long long *t = ep.trace + (size_t)blockIdx.x * 5;
      t[0] = tr0; t[1] = tr1; t[2] = tr2; t[3] = tr3; t[4] = hw;
    }
  }
#endif
}

// extent in bytes of a K x rows operand as the kernel addresses it; 0 if it does not fit a 31-bit offset
inline long operand_bytes(bool kc, long rows, long K, long ld) {
  long el = kc ? (rows - 1) * ld + K : (K - 1) * ld + rows;
  return el * 2 < 0x7fffffffL ? el * 2 : 0;
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int NSTG, bool A_KC, bool B_KC, int EPI>
int launch_dma(stp_ctx *ctx, const stp_gemm_args *a, const Epi &ep, hipStream_t s) {
  constexpr size_t smem = (size_t)NSTG * (BM + BN) * DK * 2 + 1024;      // stages, then the dump area of unused load slots
  static_assert(smem <= 160 * 1024 && smem >= (size_t)WAVES_M * WAVES_N * 32 * (BN / WAVES_N + 8) * sizeof(float), "LDS budget");
  auto kern = gemm_bf16_dma_kernel<BM, BN, WAVES_M, WAVES_N, NSTG, A_KC, B_KC, EPI>;
  static bool attr_set = false;
  if (!attr_set) {
    STP_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
    attr_set = true;
  }
  const int tiles_m = (a->M + BM - 1) / BM, tiles_n = (a->N + BN - 1) / BN;
  const long ab = operand_bytes(A_KC, a->M, a->K, a->lda), bb = operand_bytes(B_KC, a->N, a->K, a->ldb);
  hipLaunchKernelGGL(kern, dim3(tiles_m * tiles_n), dim3(64 * WAVES_M * WAVES_N), smem, s, (const bf16_t *)a->A, a->lda, (int)ab, (const bf16_t *)a->B,
                     a->ldb, (int)bb, a->M, a->N, a->K, tiles_m, tiles_n, ep);
  STP_LAUNCH_CHECK(ctx);
  return STP_OK;
}

template <int BM, int BN, int WAVES_M, int WAVES_N, bool A_KC, bool B_KC, int EPI>
int launch_cfg(stp_ctx *ctx, const stp_gemm_args *a, const Epi &ep, hipStream_t s) {
  using GA = TileGeom<BM, A_KC>;
  using GB = TileGeom<BN, B_KC>;
  constexpr size_t smem = (size_t)2 * (GA::elems + GB::elems) * sizeof(bf16_t);
  static_assert(smem <= 160 * 1024, "LDS budget");
  auto kern = gemm_bf16_kernel<BM, BN, WAVES_M, WAVES_N, A_KC, B_KC, EPI>;
  static bool attr_set = false;   // the attribute is per function; setting it twice is harmless
  if (!attr_set) {
    STP_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
    attr_set = true;
  }
  int tiles_m = (a->M + BM - 1) / BM, tiles_n = (a->N + BN - 1) / BN;
  hipLaunchKernelGGL(kern, dim3(tiles_m * tiles_n), dim3(64 * WAVES_M * WAVES_N), smem, s, (const bf16_t *)a->A, a->lda, (const bf16_t *)a->B,
                     a->ldb, a->M, a->N, a->K, tiles_m, tiles_n, ep);
  STP_LAUNCH_CHECK(ctx);
  return STP_OK;
}

// Tile choice.  A launch runs in rounds of as many workgroups as the 256 CUs hold at once (one per CU; two
// for the 128 x 128 tile, whose LDS and registers allow it), so a shape that leaves the last round
// nearly empty with big tiles can finish sooner with smaller, less efficient ones.  The estimate is
//   sum over rounds of (K/32 x t_ktile x (0.8 + 0.2 x fill) + t_fixed)
// with t_ktile the measured time of one 32-deep K-tile step of a resident workgroup on a full chip
// (microseconds, from 8192^3 runs per operand layout), fill the fraction of the round's slots in use
// (a partly filled chip leaves each workgroup more L2 and fabric bandwidth) and t_fixed the prologue +
// epilogue of a tile.  Against measured times of the layer's GEMM shapes the estimate is within
// 6 % on average and picks the fastest tile or one within 1 % of it.
// The 192 x 256 tile exists for 6144-token activations: 32 tile rows x (N / 256) columns fill the 256 CUs in
// whole rounds where the 256 x 256 tile leaves a quarter to a half of them idle; alone on the GPU it is the
// fastest tile for seven of the layer's eight token-major shapes (3-12 %).  When other streams run beside
// the GEMM (the braided block) those idle CUs are not idle and a GEMM spread over all of them only takes longer
// per tile: with `shared_gpu` the choice is made differently (first lines of pick_tile).
struct TileChoice { int bm, bn; };
inline TileChoice pick_tile(long M, long N, long K, bool a_kc, bool b_kc, bool shared_gpu) {
  struct Cfg { int bm, bn, per_cu; double t_ktile[4]; };   // t_ktile index: 2 * a_kc + b_kc; 0 = layout not built
  static const Cfg cfgs[5] = {{256, 256, 1, {0.761, 0.766, 0.756, 0.766}},
                              {192, 256, 1, {0.0, 0.0, 0.567, 0.617}},
                              {128, 256, 1, {0.432, 0.467, 0.428, 0.492}},
                              {256, 128, 1, {0.449, 0.451, 0.517, 0.496}},
                              {128, 128, 2, {0.240, 0.278, 0.251, 0.285}}};
  if (shared_gpu) {
    // Beside other streams' kernels the rounds of the estimate below mean nothing (what a round leaves idle the
    // other streams use), and what counts is the work a tile costs the compute units: the biggest tile, which
    // moves the fewest operand bytes per flop, as long as the launch still has enough workgroups to make progress
    // on its share of the machine.  Measured on nine workloads against the estimate below without the 192-row
    // tile: never more than 0.3 % behind, 1.5 - 7 % ahead on the shapes of the larger models.  A measured
    // preference (stp_gemm_tile_hint) overrides it shape by shape.
    const int opts[4][2] = {{256, 256}, {128, 256}, {256, 128}, {128, 128}};
    for (auto &o : opts)
      if (((M + o[0] - 1) / o[0]) * ((N + o[1] - 1) / o[1]) >= 96) return TileChoice{o[0], o[1]};
    return TileChoice{128, 128};
  }
  const double kt = (double)(K / DK);
  TileChoice best{256, 256};
  double best_t = 1e30;
  for (const Cfg &c : cfgs) {
    if (c.t_ktile[2 * a_kc + b_kc] == 0.0) continue;
    const long tiles = ((M + c.bm - 1) / c.bm) * ((N + c.bn - 1) / c.bn);
    const long slots = 256L * c.per_cu;
    const long full = tiles / slots, rem = tiles % slots;
    const double tk = kt * c.t_ktile[2 * a_kc + b_kc], t_fixed = 1.0 + 3.0 * (c.bm * c.bn / 65536.0);
    double t = (double)full * c.per_cu * (tk + t_fixed);
    if (rem) {
      // a partial round of the two-per-CU tile runs one workgroup per CU if it fits the 256 CUs
      const bool paired = c.per_cu == 2 && rem > 256;
      const double fill = paired ? rem / 512.0 : (rem < 256 ? rem / 256.0 : 1.0);
      t += (paired ? 2.0 : 1.0) * (tk * (0.8 + 0.2 * fill) + t_fixed);
    }
    if (t < best_t) { best_t = t; best = TileChoice{c.bm, c.bn}; }
  }
  return best;
}

template <bool A_KC, bool B_KC, int EPI>
int launch_tile(stp_ctx *ctx, const stp_gemm_args *a, const Epi &ep, hipStream_t s) {
  const bool dma_ok = a->K % DK == 0 && operand_bytes(A_KC, a->M, a->K, a->lda) > 0 && operand_bytes(B_KC, a->N, a->K, a->ldb) > 0;
  if (!dma_ok) return launch_cfg<128, 128, 2, 2, A_KC, B_KC, EPI>(ctx, a, ep, s);
  TileChoice c = pick_tile(a->M, a->N, a->K, A_KC, B_KC, ctx && ctx->concurrent);
  if (ctx && ctx->concurrent)       // a measured preference for this shape beside other streams' kernels
    for (int i = 0; i < ctx->n_tile_hints; i++) {
      const auto &hnt = ctx->tile_hint[i];
      if (hnt.M == a->M && hnt.N == a->N && hnt.K == a->K && hnt.layout == 2 * (int)A_KC + (int)B_KC) { c = TileChoice{hnt.tile_m, hnt.tile_n}; break; }
    }
  if (a->tile_m) c = TileChoice{a->tile_m, a->tile_n};
  if constexpr (A_KC) {
    // 192 rows: 6144 tokens are 32 such tiles, and 32 x (N / 256) fills the 256 compute units in whole rounds
    if (c.bm == 192 && c.bn == 256) return launch_dma<192, 256, 2, 4, DSTAGES, A_KC, B_KC, EPI>(ctx, a, ep, s);
  }
  if (c.bm == 256 && c.bn == 128) return launch_dma<256, 128, 2, 4, DSTAGES, A_KC, B_KC, EPI>(ctx, a, ep, s);
  if (c.bm == 128 && c.bn == 256) return launch_dma<128, 256, 2, 4, DSTAGES, A_KC, B_KC, EPI>(ctx, a, ep, s);
  if (c.bm == 128 && c.bn == 128) return launch_dma<128, 128, 2, 4, DSTAGES, A_KC, B_KC, EPI>(ctx, a, ep, s);
  return launch_dma<256, 256, 2, 4, DSTAGES, A_KC, B_KC, EPI>(ctx, a, ep, s);
}

template <bool A_KC, bool B_KC>
int launch_layout(stp_ctx *ctx, const stp_gemm_args *a, hipStream_t s) {
  Epi ep;
#ifdef STP_GEMM_TRACE
  ep.trace = getenv("STP_TRACE_PTR") ? (long long *)strtoull(getenv("STP_TRACE_PTR"), nullptr, 0) : nullptr;
#endif
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

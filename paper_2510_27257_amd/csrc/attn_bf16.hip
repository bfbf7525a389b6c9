// Tiled attention forward for bf16 on the CDNA4 matrix cores ("Attention(.)" of Eq. 1:
// the attention core of one TP rank, no communication).
//
// Work decomposition.  A workgroup owns 128 query rows of one (sequence, head) and ONE CHUNK of up
// to `chunk_steps` * 128 keys (chosen per launch); chunks of the same query block are merged afterwards by a small combine kernel
// (fixed order, deterministic).  Cutting the key range into chunks turns the causal triangle into
// pieces of similar size instead of workgroups whose length varies 1..seq/128.  The chunk length and the
// order in which the (block, chunk) pairs are dispatched - longest first, so that the short remainders fill
// the end of the launch - come from a host-side plan that simulates the dispatch over the 256 compute units.
// Inside a workgroup 8 waves run as 4 query sub-tiles (32 rows) x 2 key halves: per 128-key step
// waves 0-3 (group A) take keys 0..63 and waves 4-7 (group B) keys 64..127; a SIMD holds one wave of
// each group.  The two halves are merged through LDS at the end.
//
// Grouped-query attention: query head i reads key / value head i / (n / nk); only the tile addresses change.
//
// Per wave the kernel works on the TRANSPOSED score tile, S^T = K Q^T: with the 32x32x16 MFMA the
// accumulator of lane l then holds column q = l % 32, i.e. every softmax statistic (running max,
// running sum, rescale factor) is a per-lane scalar and a row reduction is an in-lane loop plus one
// cross-half shuffle.  The probabilities are already in the register layout the next MFMA wants for
// its B operand (O^T += V^T P^T), so P never touches LDS.  V^T fragments come from the V tile as it
// lies in memory ([kv][d]) through the transposing LDS read.
//
// Schedule.  A step of a wave is a matrix phase M(k) = { S(k+1) = K(k+1) Q^T ; O += V(k)^T P(k) } and
// a vector phase V(k) = { P(k) = online softmax of S(k) }, of about equal length.  In iteration k group
// A runs M(k) then V(k+1) and group B V(k) then M(k), so on every SIMD one wave feeds the matrix pipe
// while the other does the exponentials; there is one s_barrier per iteration, none between the phases.
// K and V tiles (128 keys x D) go global -> LDS directly (buffer_load ... lds), K and V each in a ring
// of two tiles.  Tile K(k+2) replaces K(k) and V(k+1) replaces V(k-1); both are issued at the top of
// iteration k, when every wave is done with the tiles they overwrite, and waited for (vmcnt(0) + the
// barrier) at the top of iteration k+1, where they are first used.  A direct-to-LDS wave instruction fills
// 1 KB contiguously, so rows cannot be padded; bank conflicts are avoided by an XOR permutation of
// the 16-byte chunks of a row, applied on the global side and undone in the fragment addresses:
//   K tile [key][D]: chunk c of row r in slot c ^ ((r / RPB) & (CPR-1))        (16-byte fragment reads)
//   V tile [key][D]: chunk c of row r in slot c ^ (4 * ((r & 3) / RPB))        (ds_read_b64_tr_b16 reads)
// with CPR = D/8 chunks per row and RPB = 128/D rows per 256 bytes.  Fragment reads are inline assembly
// with explicit waits, software-pipelined one group of MFMAs ahead.
#include "common.h"
#include "lds_dma.h"
#include <type_traits>
#include <vector>
#include <algorithm>
#include <queue>
#include <functional>
#include <cstring>

namespace {

constexpr int QB = 128;    // query rows per workgroup
constexpr int KSTEP = 128; // keys per step (64 per wave half)
constexpr float LN2 = 0.69314718055994531f;

template <int D> struct AttnGeom {
  static constexpr int RB = D * 2;               // bytes per tile row
  static constexpr int CPR = D / 8;              // 16-byte chunks per row
  static constexpr int RPB = 256 / RB;           // rows per 256 bytes (one pass over the 64 banks)
  static constexpr int RPI = 64 / CPR;           // tile rows covered by one direct-to-LDS wave instruction
  static constexpr int NLD = KSTEP / RPI / 8;    // such instructions per wave per tile
  static constexpr int TILE = KSTEP * RB;        // bytes of a K or V tile
  static constexpr int piece_floats = QB * D + 2 * QB;   // partial O, then m, then l
};

// number of 128-key steps a query block needs
__host__ __device__ inline int attn_steps(int qb, int seq, int causal) {
  int kv_end = causal ? (seq < qb * QB + QB ? seq : qb * QB + QB) : seq;
  return (kv_end + KSTEP - 1) / KSTEP;
}

// ---- fragment reads (results valid after lds_wait + lds_tie) ----
// K fragments of sub-block JB (32 keys), d-steps 4*SG .. 4*SG+3: A operand, lane supplies key row lr, d = 16 s + 8 lg ..
template <int D, int JB, int SG>
__device__ __forceinline__ void read_k(u32x4_t (&buf)[4], const unsigned (&kaddr)[D / 16], unsigned tile) {
  constexpr int OFF = JB * 32 * AttnGeom<D>::RB;
  buf[0] = lds_read_b128<OFF>(kaddr[4 * SG + 0] + tile);
  buf[1] = lds_read_b128<OFF>(kaddr[4 * SG + 1] + tile);
  buf[2] = lds_read_b128<OFF>(kaddr[4 * SG + 2] + tile);
  buf[3] = lds_read_b128<OFF>(kaddr[4 * SG + 3] + tile);
}
// V^T fragments of keys 32 JB + 16 T .. +15 for the D/32 blocks of 32 output columns
template <int D, int JB, int T>
__device__ __forceinline__ void read_v(u32x4_t (&buf)[4], const unsigned (&vaddr)[D / 32], unsigned tile) {
  constexpr int RB = AttnGeom<D>::RB, OFF = (32 * JB + 16 * T) * RB;
  buf[0] = lds_read_tr16<OFF, 8 * RB>(vaddr[0] + tile);
  buf[1] = lds_read_tr16<OFF, 8 * RB>(vaddr[1] + tile);
  if constexpr (D == 128) {
    buf[2] = lds_read_tr16<OFF, 8 * RB>(vaddr[2] + tile);
    buf[3] = lds_read_tr16<OFF, 8 * RB>(vaddr[3] + tile);
  }
}
template <int D, int SG>
__device__ __forceinline__ void mfma_qk(f32x16_t &sc, const u32x4_t (&buf)[4], const bf16x8_t (&qf)[D / 16]) {
#pragma unroll
  for (int i = 0; i < 4; i++)
    sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, buf[i]), qf[4 * SG + i], sc, 0, 0, 0);
}
template <int D>
__device__ __forceinline__ void mfma_pv(f32x16_t (&o)[D / 32], const u32x4_t (&buf)[4], bf16x8_t pf) {
#pragma unroll
  for (int db = 0; db < D / 32; db++)
    o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, buf[db]), pf, o[db], 0, 0, 0);
}

template <int D>
__global__ __launch_bounds__(512) void attn_fwd_bf16_kernel(const bf16_t *__restrict__ qkv, float *__restrict__ part,
                                                            bf16_t *__restrict__ out, float *__restrict__ lse_out, int seq,
                                                            int n, int nk, int causal, int max_chunks, int chunk_steps, float scale_log2,
                                                            int n_items, stp_attn_order ord
#ifdef STP_ATTN_TRACE
                                                            , long long *trace
#endif
                                                            ) {
  using G = AttnGeom<D>;
  static_assert(D == 64 || D == 128, "head dimension");
#ifdef STP_ATTN_TRACE
  const long long tr0 = wall_clock64();
#endif
  constexpr int RB = G::RB, CPR = G::CPR, RPB = G::RPB, RPI = G::RPI, NLD = G::NLD, TILE = G::TILE;
  constexpr int KREADS = 4, VREADS = 2 * (D / 32);   // LDS operations of one fragment group
  extern __shared__ __attribute__((aligned(1024))) char smem_raw[];   // K ring [2][TILE], V ring [2][TILE]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lr = lane & 31, lg = lane >> 5;
  const int qsub = wave & 3, half = wave >> 2;
  const int nqb = (seq + QB - 1) / QB;
  // the workgroup's (query block, chunk): from the launch's work order (grid = heads x items), or, without
  // one, from a grid of blocks x chunks x heads with the late query blocks, which own the most chunks, first
  const int item = n_items ? ord.item[blockIdx.y] : 0;
  const int qb = n_items ? (item & 0xfff) : nqb - 1 - (int)blockIdx.x;
  const int chunk = n_items ? (item >> 12) : (int)blockIdx.y;
  const int bz = n_items ? blockIdx.x : blockIdx.z;
  const int head = bz % n, b = bz / n;
  const int nsteps = attn_steps(qb, seq, causal);
  const int s_begin = chunk * chunk_steps, s_end = min(nsteps, s_begin + chunk_steps);
  if (s_begin >= nsteps) return;
  const int ns = s_end - s_begin;

  const int a = n * D;
  const int ld = (n + 2 * nk) * D;              // a qkv row: n Q heads, nk K heads, nk V heads
  const int kcol = a + (head / (n / nk)) * D, vcol = kcol + nk * D;   // this head's key / value head
  const bf16_t *bbase = qkv + (size_t)b * seq * ld;           // this sequence's [seq][3a] block
  const int q_wave0 = qb * QB + qsub * 32;
  const int qg = q_wave0 + lr;                  // this lane's query row
  const int q_ld = min(qg, seq - 1);            // clamp so that tail lanes read valid memory

  // Q fragments: B operand, lane supplies row q, k = d index 16*s + 8*lg .. +7
  bf16x8_t qf[D / 16];
#pragma unroll
  for (int s = 0; s < D / 16; s++)
    qf[s] = *reinterpret_cast<const bf16x8_t *>(bbase + (size_t)q_ld * ld + head * D + 16 * s + 8 * lg);

  // ---- direct-to-LDS loads of this wave: instruction I = wave * NLD + j covers tile rows I*RPI .. +RPI-1
  const __amdgpu_buffer_rsrc_t rs =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(bbase), 0, (int)min((size_t)seq * ld * 2, (size_t)0x7fffffff), 0x00020000);
  // lane's byte offset = min(row offset, last row's) + column offset; the row offset is this lane's row within the
  // wave's first instruction (a register) plus a wave-uniform part (step, instruction), so a load costs three
  // vector instructions and no multiplication, and its LDS target is computed on the scalar unit
  const int wave_s = __builtin_amdgcn_readfirstlane(wave);     // same value, known to be wave-uniform
  const unsigned row_bytes = (unsigned)ld * 2u, max_rowoff = (unsigned)(seq - 1) * row_bytes;
  const unsigned ld_rowoff0 = (unsigned)(wave * NLD * RPI + lane / CPR) * row_bytes;
  unsigned ld_kcol[NLD], ld_vcol[NLD];          // byte offset within a qkv row of the chunk this lane fetches
#pragma unroll
  for (int j = 0; j < NLD; j++) {
    const int row = (wave * NLD + j) * RPI + lane / CPR, slot = lane % CPR;
    ld_kcol[j] = (unsigned)(kcol + (slot ^ ((row / RPB) & (CPR - 1))) * 8) * 2u;
    ld_vcol[j] = (unsigned)(vcol + (slot ^ (4 * ((row & 3) / RPB))) * 8) * 2u;
  }
  // load j (0 .. NLD-1) of the K or V tile of local step k, into ring slot k & 1; rows past the end of the
  // sequence read its last row
  auto issue_one = [&](int k, bool is_v, int j) {
    char *dst = smem_raw + (is_v ? 2 * TILE : 0) + (k & 1) * TILE + (wave_s * NLD + j) * 1024;
    const unsigned uni = (unsigned)((s_begin + k) * KSTEP + j * RPI) * row_bytes;
    const unsigned rowoff = min(ld_rowoff0 + uni, max_rowoff);
    dma_load16(rs, dst, rowoff + (is_v ? ld_vcol[j] : ld_kcol[j]), 0);
  };
  auto issue_tile = [&](int k, bool is_v) {
#pragma unroll
    for (int j = 0; j < NLD; j++) issue_one(k, is_v, j);
  };

  // ---- fragment addresses within a tile (this wave's 64-key half)
  const unsigned lds0 = (unsigned)(size_t)(const __attribute__((address_space(3))) char *)smem_raw;
  unsigned kaddr[D / 16], vaddr[D / 32];
  {
    const int row = half * 64 + lr;
#pragma unroll
    for (int s = 0; s < D / 16; s++) kaddr[s] = lds0 + row * RB + (((2 * s + lg) ^ ((row / RPB) & (CPR - 1))) * 16);
    // lane reads 4 consecutive d of key kbase + 4 lg + (lane&15)/4 (and of that key + 8): the k-slot order of P^T
    const int key = half * 64 + 4 * lg + ((lane & 15) >> 2);
#pragma unroll
    for (int db = 0; db < D / 32; db++) {
      const int col = 32 * db + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
      vaddr[db] = lds0 + 2 * TILE + key * RB + (((col >> 3) ^ (4 * ((key & 3) / RPB))) * 16) + (col & 7) * 2;
    }
  }

  f32x16_t o[D / 32];
#pragma unroll
  for (int i = 0; i < D / 32; i++)
#pragma unroll
    for (int v = 0; v < 16; v++) o[i][v] = 0.f;
  float m = -INFINITY, l = 0.f;
  f32x16_t sc0, sc1;                 // S^T of the step in flight: keys 0..31 and 32..63 of this wave's half
  bf16x8_t pf00, pf01, pf10, pf11;   // P^T of the step whose PV is pending: [sub-block][16-key half]
#pragma unroll
  for (int i = 0; i < 8; i++) { pf00[i] = (bf16_t)0.f; pf01[i] = (bf16_t)0.f; pf10[i] = (bf16_t)0.f; pf11[i] = (bf16_t)0.f; }

  // wave-uniform: does local step k hold a key this wave's queries may attend to?
  auto active = [&](int k) {
    const int kv0 = (s_begin + k) * KSTEP + half * 64;
    return kv0 < seq && (!causal || kv0 <= q_wave0 + 31);
  };

#define STP_SB() __builtin_amdgcn_sched_barrier(0)
  // S(kn) = K(kn) Q^T
  auto qk_only = [&](int kn) {
    const unsigned kt = (kn & 1) * TILE;
    u32x4_t fa[4], fb[4];
#pragma unroll
    for (int v = 0; v < 16; v++) { sc0[v] = 0.f; sc1[v] = 0.f; }
    read_k<D, 0, 0>(fa, kaddr, kt);
    if constexpr (D == 128) {
      read_k<D, 0, 1>(fb, kaddr, kt); lds_wait<KREADS>(); lds_tie(fa); mfma_qk<D, 0>(sc0, fa, qf); STP_SB();
      read_k<D, 1, 0>(fa, kaddr, kt); lds_wait<KREADS>(); lds_tie(fb); mfma_qk<D, 1>(sc0, fb, qf); STP_SB();
      read_k<D, 1, 1>(fb, kaddr, kt); lds_wait<KREADS>(); lds_tie(fa); mfma_qk<D, 0>(sc1, fa, qf); STP_SB();
      lds_wait<0>(); lds_tie(fb); mfma_qk<D, 1>(sc1, fb, qf); STP_SB();
    } else {
      read_k<D, 1, 0>(fb, kaddr, kt); lds_wait<KREADS>(); lds_tie(fa); mfma_qk<D, 0>(sc0, fa, qf); STP_SB();
      lds_wait<0>(); lds_tie(fb); mfma_qk<D, 0>(sc1, fb, qf); STP_SB();
    }
  };
  // O^T += V(k)^T P^T
  auto pv_only = [&](int k) {
    const unsigned vt = (k & 1) * TILE;
    u32x4_t fa[4], fb[4];
    read_v<D, 0, 0>(fa, vaddr, vt);
    read_v<D, 0, 1>(fb, vaddr, vt); lds_wait<VREADS>(); lds_tie(fa); mfma_pv<D>(o, fa, pf00); STP_SB();
    read_v<D, 1, 0>(fa, vaddr, vt); lds_wait<VREADS>(); lds_tie(fb); mfma_pv<D>(o, fb, pf01); STP_SB();
    read_v<D, 1, 1>(fb, vaddr, vt); lds_wait<VREADS>(); lds_tie(fa); mfma_pv<D>(o, fa, pf10); STP_SB();
    lds_wait<0>(); lds_tie(fb); mfma_pv<D>(o, fb, pf11); STP_SB();
  };
  // both, as one software pipeline (the common case).  With `defer` the wave's direct-to-LDS loads of this
  // iteration (K(k+2) if ld_k, V(k+1) if ld_v) are issued one at a time behind the MFMA groups, whose
  // execution covers the time the address unit holds the wave, instead of in a burst before them.
  auto qk_pv = [&](int kn, int k, bool ld_k, bool ld_v) {
    const unsigned kt = (kn & 1) * TILE, vt = (k & 1) * TILE;
    u32x4_t fa[4], fb[4];
#pragma unroll
    for (int v = 0; v < 16; v++) { sc0[v] = 0.f; sc1[v] = 0.f; }
    // the 2 * NLD loads are spread over the first 2 * NLD of the 8 (D = 128) or 6 (D = 64) groups
#define STP_LD(g)                                                        \
    do {                                                                 \
      if ((g) < NLD) { if (ld_k) issue_one(k + 2, false, (g)); }         \
      else if ((g) < 2 * NLD) { if (ld_v) issue_one(k + 1, true, (g) - NLD); } \
      STP_SB();                                                          \
    } while (0)
    read_k<D, 0, 0>(fa, kaddr, kt);
    if constexpr (D == 128) {
      read_k<D, 0, 1>(fb, kaddr, kt); lds_wait<KREADS>(); lds_tie(fa); mfma_qk<D, 0>(sc0, fa, qf); STP_SB(); STP_LD(0);
      read_k<D, 1, 0>(fa, kaddr, kt); lds_wait<KREADS>(); lds_tie(fb); mfma_qk<D, 1>(sc0, fb, qf); STP_SB(); STP_LD(1);
      read_k<D, 1, 1>(fb, kaddr, kt); lds_wait<KREADS>(); lds_tie(fa); mfma_qk<D, 0>(sc1, fa, qf); STP_SB(); STP_LD(2);
      read_v<D, 0, 0>(fa, vaddr, vt); lds_wait<VREADS>(); lds_tie(fb); mfma_qk<D, 1>(sc1, fb, qf); STP_SB(); STP_LD(3);
      read_v<D, 0, 1>(fb, vaddr, vt); lds_wait<VREADS>(); lds_tie(fa); mfma_pv<D>(o, fa, pf00); STP_SB(); STP_LD(4);
      read_v<D, 1, 0>(fa, vaddr, vt); lds_wait<VREADS>(); lds_tie(fb); mfma_pv<D>(o, fb, pf01); STP_SB(); STP_LD(5);
      read_v<D, 1, 1>(fb, vaddr, vt); lds_wait<VREADS>(); lds_tie(fa); mfma_pv<D>(o, fa, pf10); STP_SB(); STP_LD(6);
      lds_wait<0>(); lds_tie(fb); mfma_pv<D>(o, fb, pf11); STP_SB(); STP_LD(7);
    } else {
      read_k<D, 1, 0>(fb, kaddr, kt); lds_wait<KREADS>(); lds_tie(fa); mfma_qk<D, 0>(sc0, fa, qf); STP_SB(); STP_LD(0);
      read_v<D, 0, 0>(fa, vaddr, vt); lds_wait<VREADS>(); lds_tie(fb); mfma_qk<D, 0>(sc1, fb, qf); STP_SB(); STP_LD(1);
      read_v<D, 0, 1>(fb, vaddr, vt); lds_wait<VREADS>(); lds_tie(fa); mfma_pv<D>(o, fa, pf00); STP_SB(); STP_LD(2);
      read_v<D, 1, 0>(fa, vaddr, vt); lds_wait<VREADS>(); lds_tie(fb); mfma_pv<D>(o, fb, pf01); STP_SB(); STP_LD(3);
      read_v<D, 1, 1>(fb, vaddr, vt); lds_wait<VREADS>(); lds_tie(fa); mfma_pv<D>(o, fa, pf10); STP_SB();
      lds_wait<0>(); lds_tie(fb); mfma_pv<D>(o, fb, pf11); STP_SB();
    }
#undef STP_LD
  };

  // P(k) = online softmax of S(k) in the log2 domain; accumulator v of lane l is key
  // kv0 + 32*jb + 8*(v/4) + 4*(l/32) + v%4, query l%32
  auto softmax_impl = [&](int k, auto masked) {
    constexpr bool MASK = decltype(masked)::value;
    const int kv0 = (s_begin + k) * KSTEP + half * 64;
    // raw scores are kept; the 1/sqrt(d) log2(e) factor is folded into the exponent's FMA
    auto mask_max = [&](f32x16_t &sc, int jb, float mx) {
      if constexpr (MASK) {
#pragma unroll
        for (int v = 0; v < 16; v++) {
          const int kv = kv0 + 32 * jb + 8 * (v >> 2) + 4 * lg + (v & 3);
          sc[v] = ((causal && kv > qg) || kv >= seq) ? -INFINITY : sc[v];
        }
      }
#pragma unroll
      for (int v = 0; v < 16; v++) mx = fmaxf(mx, sc[v]);
      return mx;
    };
    float mx = mask_max(sc0, 0, -INFINITY);
    mx = mask_max(sc1, 1, mx);
    mx = fmaxf(mx, other_half(mx)) * scale_log2;      // scale > 0: max and scaling commute
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
    float rs = 0.f;
    // k-slot i of lane-half g in the PV step (jb, t) is key 32*jb + 16*t + 8*(i/4) + 4*g + i%4
    auto exp_pack = [&](const f32x16_t &sc, bf16x8_t &p0, bf16x8_t &p1) {
#pragma unroll
      for (int v = 0; v < 16; v++) {
        const float p = __builtin_amdgcn_exp2f(fmaf(sc[v], scale_log2, neg_ref));
        rs += p;
        if (v < 8) p0[v] = (bf16_t)p; else p1[v - 8] = (bf16_t)p;
      }
    };
    exp_pack(sc0, pf00, pf01);
    exp_pack(sc1, pf10, pf11);
    rs += other_half(rs);
    l += rs;
  };
  // only a step that touches the causal diagonal or the end of the sequence needs the mask
  auto softmax = [&](int k) {
    const int kv0 = (s_begin + k) * KSTEP + half * 64;
    if ((causal && kv0 + 63 > q_wave0) || (kv0 + 64 > seq)) softmax_impl(k, std::true_type{});
    else softmax_impl(k, std::false_type{});
  };

  // ---- main loop.  Iteration k uses tiles K(k+1) and V(k).  At its top every wave's loads have landed
  // (vmcnt(0) + barrier) and every wave is done with K(k) and V(k-1), whose slots take K(k+2) and V(k+1).
  // Group A runs M(k) then V(k+1), group B V(k) then M(k): the matrix work of one wave of a SIMD
  // coincides with the vector work of the other without a barrier in between.
  const bool last_active = active(ns - 1);      // only the last step of a chunk can be masked out for a wave
  auto vector_phase = [&](int k) {
    if (k >= 0 && k < ns && (k < ns - 1 || last_active)) softmax(k);
  };
  issue_tile(0, false);
  issue_tile(0, true);
  if (ns > 1) {
    issue_tile(1, false);
    asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(2 * NLD) : "memory");
  } else {
    asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(NLD) : "memory");
  }
#ifdef STP_ATTN_TRACE
  const long long tr1 = wall_clock64();
#endif
  for (int k = -1; k < ns; k++) {
    const bool do_qk = k + 1 < ns && (k + 1 < ns - 1 || last_active), do_pv = k >= 0 && (k < ns - 1 || last_active);
    const bool ld_k = k >= 0 && k + 2 < ns, ld_v = k >= 0 && k + 1 < ns;
    // group A starts with the matrix phase: its loads ride behind the MFMA groups
    const bool defer = half == 0 && do_qk && do_pv;
    if (k >= 0) {
      STP_SB();
      asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
      STP_SB();
      if (!defer) {
        if (ld_k) issue_tile(k + 2, false);
        if (ld_v) issue_tile(k + 1, true);
      }
    }
    if (half == 1) vector_phase(k);
    if (do_qk && do_pv) qk_pv(k + 1, k, defer && ld_k, defer && ld_v);
    else if (do_qk) qk_only(k + 1);
    else if (do_pv) pv_only(k);
    if (half == 0) vector_phase(k + 1);
  }
#undef STP_SB
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
#ifdef STP_ATTN_TRACE
  const long long tr2 = wall_clock64();
#endif

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
    if (qg < seq && nsteps <= chunk_steps) {
      // the query block has this one chunk: its rows are final, so they go to the output (and the log-sum-exp)
      // directly and the combine kernel leaves them alone
      const float inv = 1.0f / l;
      bf16_t *op = out + ((size_t)b * seq + qg) * a + head * D;
      typedef bf16_t bf16x4_t __attribute__((ext_vector_type(4)));
#pragma unroll
      for (int i = 0; i < D / 32; i++)
#pragma unroll
        for (int j = 0; j < 4; j++) {
          bf16x4_t w;
#pragma unroll
          for (int r = 0; r < 4; r++) {
            const int v = 4 * j + r;
            w[r] = (bf16_t)((o[i][v] * ea + red[(qsub * (D / 2) + i * 16 + v) * 64 + lane] * eb) * inv);
          }
          *reinterpret_cast<bf16x4_t *>(op + 32 * i + 8 * j + 4 * lg) = w;
        }
      if (lg == 0) lse_out[((size_t)b * n + head) * seq + qg] = (M + log2f(l)) * LN2;
    } else if (qg < seq) {
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
#ifdef STP_ATTN_TRACE
  if (trace) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    const long long tr3 = wall_clock64();
    if (tid == 0) {
      unsigned hw, xcc;
      asm volatile("s_getreg_b32 %0, hwreg(HW_REG_HW_ID)" : "=s"(hw));
      asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
      long long *t = trace + ((size_t)blockIdx.y * gridDim.x + blockIdx.x) * 8;
      t[0] = tr0; t[1] = tr1; t[2] = tr2; t[3] = tr3; t[4] = hw; t[5] = xcc; t[6] = ns; t[7] = 1;
    }
  }
#endif
}

// out[q, :] = sum_c O_c e^{m_c - M} / sum_c l_c e^{m_c - M}; lse = (M + log2 L) ln 2.  One wave per (token, head).
template <int D>
__global__ __launch_bounds__(256) void attn_fwd_combine_kernel(const float *__restrict__ part, bf16_t *__restrict__ out,
                                                               float *__restrict__ lse, int seq, int n, int mbsz, int causal,
                                                               int max_chunks, int chunk_steps, int q_first) {
  using G = AttnGeom<D>;
  const int lane = threadIdx.x & 63;
  const size_t w = blockIdx.x * (size_t)4 + (threadIdx.x >> 6);
  const int rows = seq - q_first;             // rows below q_first belong to one-chunk blocks, which the main kernel finished
  if (w >= (size_t)mbsz * n * rows) return;
  const int q = q_first + w % rows, head = (w / rows) % n, b = w / ((size_t)rows * n);
  const int nqb = (seq + QB - 1) / QB, qb = q / QB, qloc = q % QB;
  const int nch = (attn_steps(qb, seq, causal) + chunk_steps - 1) / chunk_steps;
  if (nch <= 1) return;
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

// the plan of the forward kernel for this shape (block x = query block x)
inline const stp_attn_plan *fwd_plan(stp_ctx *ctx, const stp_layer_desc *d) {
  const int nqb = (d->seq + QB - 1) / QB;
  std::vector<int> steps(nqb);
  for (int x = 0; x < nqb; x++) steps[x] = attn_steps(x, d->seq, d->causal);
  return stp_attn_plan_get(ctx, 0, d, nqb, steps.data(), d->heads_local * d->mbsz);
}

template <int D>
int launch_fwd(stp_ctx *ctx, const stp_layer_desc *d, const void *qkv, void *out, float *lse, float *ws, size_t ws_bytes,
               hipStream_t s) {
  using G = AttnGeom<D>;
  constexpr size_t smem = (size_t)4 * G::TILE;   // K ring and V ring of two tiles each
  static_assert(smem >= (size_t)(4 * (D / 2) * 64 + 4 * 2 * 32) * sizeof(float), "merge area fits");
  static_assert(smem <= 160 * 1024, "LDS budget");
  auto kern = attn_fwd_bf16_kernel<D>;
  static bool attr_set = false;
  if (!attr_set) {
    STP_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
    attr_set = true;
  }
  if ((size_t)d->seq * stp_qkv_width(d) * sizeof(bf16_t) > (size_t)0x7fffffff)
    return stp_fail(ctx, STP_ESHAPE, "attention forward: one sequence of QKV must span less than 2 GiB%s");
  const int nqb = (d->seq + QB - 1) / QB;
  const stp_attn_plan *plan = fwd_plan(ctx, d);
  const int chunk_steps = plan->chunk_steps, max_chunks = plan->max_chunks;
  const size_t need = (size_t)d->mbsz * d->heads_local * nqb * max_chunks * G::piece_floats * sizeof(float);
  if (!ws || ws_bytes < need)
    return stp_fail(ctx, STP_ENOSPACE, "attention forward: workspace lane too small%s (need %ld bytes)", "", (long)need);
  const dim3 grid = plan->n_items ? dim3(d->heads_local * d->mbsz, plan->n_items) : dim3(nqb, max_chunks, d->heads_local * d->mbsz);
  const dim3 block(512);
  float scale_log2 = 1.4426950408889634f / sqrtf((float)D);
  hipLaunchKernelGGL(kern, grid, block, smem, s, (const bf16_t *)qkv, ws, (bf16_t *)out, lse, d->seq, d->heads_local, stp_kv_heads(d), d->causal, max_chunks, chunk_steps,
                     scale_log2, plan->n_items, plan->order
#ifdef STP_ATTN_TRACE
                     , getenv("STP_TRACE_PTR") ? (long long *)strtoull(getenv("STP_TRACE_PTR"), nullptr, 0) : (long long *)nullptr
#endif
                     );
  STP_LAUNCH_CHECK(ctx);
  // query blocks with a single chunk were finished by the main kernel; with the causal mask they are the first ones
  int qb_first = 0;
  while (qb_first < nqb && attn_steps(qb_first, d->seq, d->causal) <= chunk_steps) qb_first++;
  if (qb_first < nqb) {
    const int q_first = qb_first * QB;
    size_t waves = (size_t)d->mbsz * d->heads_local * (d->seq - q_first);
    hipLaunchKernelGGL(attn_fwd_combine_kernel<D>, dim3((waves + 3) / 4), dim3(256), 0, s, ws, (bf16_t *)out, lse, d->seq,
                       d->heads_local, d->mbsz, d->causal, max_chunks, chunk_steps, q_first);
    STP_LAUNCH_CHECK(ctx);
  }
  return STP_OK;
}

}  // namespace

const stp_attn_plan *stp_attn_plan_for(stp_ctx *ctx, const stp_layer_desc *d, int kind) {
  return kind == 0 ? fwd_plan(ctx, d) : stp_attn_bwd_plan_for(ctx, d, kind);
}

size_t stp_attn_fwd_ws_bytes(const stp_layer_desc *d) {
  const int nqb = (d->seq + QB - 1) / QB;
  const int max_chunks = fwd_plan(nullptr, d)->max_chunks;
  return (size_t)d->mbsz * d->heads_local * nqb * max_chunks * (QB * d->head_dim + 2 * QB) * sizeof(float);
}

int stp_launch_attn_fwd_bf16(stp_ctx *ctx, const stp_layer_desc *d, const void *qkv, void *out, float *lse, float *ws,
                             size_t ws_bytes, hipStream_t s) {
  if (d->head_dim == 128) return launch_fwd<128>(ctx, d, qkv, out, lse, ws, ws_bytes, s);
  if (d->head_dim == 64) return launch_fwd<64>(ctx, d, qkv, out, lse, ws, ws_bytes, s);
  return stp_fail(ctx, STP_ESHAPE, "bf16 attention needs head_dim 64 or 128%s");
}

// Cost of a workgroup of the chunked kernels in microseconds (index: 0 forward, 1 dkv, 2 dq): start and end of a
// workgroup (first tiles, the merge of the wave halves, the partial result) and one step of its main loop; fitted
// to measured kernel times over chunk lengths 8 .. 32 (16 .. 64 for dkv) at 4 and 10 heads x 128, seq 4096 and
// 6144, causal, and 16 heads, seq 1024, not causal: the estimate is within 6 - 8 % (rms) and its choice is the
// fastest chunk length measured, or within 3 % of it.
static const double kFixedUs[3] = {11.5, 12.0, 12.0}, kStepUs[3] = {1.75, 1.90, 2.65};
// compute units a chunked attention launch counts on inside a braided block (measured: 96 gives the fastest block on
// the 4-head and 10-head workloads, 0.3 - 2.5 % ahead of planning for all 256; 32 is 4 - 8 % behind)
#define STP_ATTN_SHARED_CUS 96

namespace {

// Time of a launch whose workgroups, in the given order, each go to the compute unit that is free first
// (256 of them, one workgroup each): fixed + per_step * steps per workgroup, every length `zcount` times.
double plan_makespan(const std::vector<int> &lens, int zcount, double fixed, double per_step, int cus) {
  // many (head, sequence) pairs: 16 of them on a proportionally smaller machine give the same picture
  // and keep the planning time bounded
  if (zcount > 16) { cus = std::max(1, cus * 16 / zcount); zcount = 16; }
  std::priority_queue<double, std::vector<double>, std::greater<double>> cu;
  for (int i = 0; i < cus; i++) cu.push(0.0);
  double end = 0.0;
  for (int len : lens)
    for (int z = 0; z < zcount; z++) {
      const double t = cu.top() + fixed + per_step * len;
      cu.pop();
      cu.push(t);
      end = std::max(end, t);
    }
  return end;
}

// cus: the compute units the launch can count on (all 256 when it has the GPU to itself; fewer inside a braided
// block, where longer chunks, i.e. fewer workgroups with their fixed cost, win because the other streams' kernels
// fill what an uneven end of the launch leaves idle); min_chunk: never shorter than this
void plan_make(int kind, int nblocks, const int *steps, int zcount, stp_attn_plan *plan, int cus = 256, int min_chunk = 0) {
  const double *fixed_us = kFixedUs, *step_us = kStepUs;
  int max_steps = 1;
  for (int x = 0; x < nblocks; x++) max_steps = std::max(max_steps, steps[x]);
  // a block is never cut into more than 8 pieces (bounds the workspace and fits the table's 3 chunk bits)
  const int lo = std::max((max_steps + 7) / 8, std::min(max_steps, 4));
  int best_c = max_steps;
  double best_t = 1e30;
  std::vector<int> lens;
  const int stride = std::max(1, (max_steps - lo) / 48);      // at most about 48 candidates
  for (int c = lo; c <= max_steps; c += stride) {
    if (c < min_chunk) continue;
    lens.clear();
    for (int x = 0; x < nblocks; x++) {
      for (int k = 0; k < steps[x] / c; k++) lens.push_back(c);
      if (steps[x] % c) lens.push_back(steps[x] % c);
    }
    std::sort(lens.begin(), lens.end(), std::greater<int>());
    const double t = plan_makespan(lens, zcount, fixed_us[kind], step_us[kind], cus);
    if (t < best_t * 0.995) { best_t = t; best_c = c; }      // a longer chunk has to win by half a percent
  }
  plan->chunk_steps = best_c;
  plan->max_chunks = (max_steps + best_c - 1) / best_c;
  // the (block, chunk) pairs, longest first; equal lengths keep the later blocks first
  struct Item { int len, block, chunk; };
  std::vector<Item> items;
  for (int x = nblocks - 1; x >= 0; x--)
    for (int k = 0; k * best_c < steps[x]; k++) items.push_back({std::min(best_c, steps[x] - k * best_c), x, k});
  std::stable_sort(items.begin(), items.end(), [](const Item &u, const Item &v) { return u.len > v.len; });
  plan->n_items = 0;
  if (items.size() <= STP_ATTN_ORDER_CAP && nblocks <= 4096 && plan->max_chunks <= 8) {
    plan->n_items = (int)items.size();
    for (size_t i = 0; i < items.size(); i++) plan->order.item[i] = (uint16_t)(items[i].block | (items[i].chunk << 12));
  }
}

}  // namespace

double stp_attn_item_cost(int kind, int len) { return kFixedUs[kind] + kStepUs[kind] * len; }

stp_attn_plan *stp_attn_plan_slot(stp_ctx *ctx, const int key[8], bool *hit) {
  static thread_local stp_attn_plan scratch_of_kind[4];
  stp_attn_plan *p = &scratch_of_kind[(key[0] - 1) & 3];
  *hit = false;
  if (ctx) {
    for (int i = 0; i < ctx->attn_plan_n; i++)
      if (memcmp(ctx->attn_plan[i].key, key, 8 * sizeof(int)) == 0) { *hit = true; return &ctx->attn_plan[i]; }
    if (ctx->attn_plan_n < STP_ATTN_PLAN_CACHE) p = &ctx->attn_plan[ctx->attn_plan_n++];
    else { p = &ctx->attn_plan[ctx->attn_plan_next]; ctx->attn_plan_next = (ctx->attn_plan_next + 1) % STP_ATTN_PLAN_CACHE; }
  } else if (memcmp(p->key, key, 8 * sizeof(int)) == 0) {
    *hit = true;
    return p;
  }
  memcpy(p->key, key, 8 * sizeof(int));
  return p;
}

const stp_attn_plan *stp_attn_plan_get(stp_ctx *ctx, int kind, const stp_layer_desc *d, int nblocks, const int *steps, int zcount) {
  const bool shared = ctx && ctx->concurrent;
  const int key[8] = {kind + 1 + (shared ? 16 : 0), d->seq, d->causal, d->heads_local, stp_kv_heads(d), d->mbsz, d->head_dim, nblocks};
  bool hit;
  stp_attn_plan *p = stp_attn_plan_slot(ctx, key, &hit);
  if (hit) return p;
  if (!shared) { plan_make(kind, nblocks, steps, zcount, p); return p; }
  // inside a block: plan for a share of the machine, never with shorter chunks than alone (the workspace is sized
  // by the lone plan's chunk count)
  stp_attn_plan alone;
  plan_make(kind, nblocks, steps, zcount, &alone);
  plan_make(kind, nblocks, steps, zcount, p, STP_ATTN_SHARED_CUS, alone.chunk_steps);
  return p;
}

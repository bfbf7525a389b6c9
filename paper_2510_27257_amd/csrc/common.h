// Internal helpers shared by the HIP translation units of libstp.so.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include "stp.h"

typedef __bf16 bf16_t;
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef short s16x8_t __attribute__((ext_vector_type(8)));

#define STP_MAX_LAYER_EVENTS 4096

// Work plan of a chunked attention kernel (forward, dq, dkv).  A workgroup owns one chunk of up to chunk_steps
// steps of one block (a query block, or a key block for dkv); `order` lists the (block, chunk) pairs, longest
// first, and the grid is (heads, n_items) so that the dispatcher, which hands out workgroups in grid order,
// starts the long ones first and fills the tail of the launch with the short ones.  item = block | chunk << 12.
// n_items = 0 (more pairs than the table holds): the grid is blocks x max_chunks x heads and a workgroup
// reads its pair from its grid position.
#define STP_ATTN_ORDER_CAP 1024
struct stp_attn_order { uint16_t item[STP_ATTN_ORDER_CAP]; };
struct stp_attn_plan {
  int key[8];          // what the plan was made for (cache tag)
  int chunk_steps, max_chunks, n_items;
  stp_attn_order order;
};
#define STP_ATTN_PLAN_CACHE 12

#define STP_TILE_HINTS 96
struct stp_ctx {
  int device;
  char err[512];
  char *ws;          // caller-supplied workspace (device)
  size_t ws_bytes;
  // End-of-step events of the three braid streams for the last two steps (generation = step parity), the stream
  // each was recorded on, and what the last step touched: its forward microbatch and, per microbatch, whether it
  // held B or W work.  A step waits for all of the step before last and, of the last one, only for the streams
  // whose work it depends on.
  hipEvent_t ev_step[2][3];
  hipStream_t ev_stream[2][3];
  int ev_alias[2][3];               // index of the event that stands for stream i (streams passed twice share one)
  int ev_valid[2], ev_gen;          // ev_gen: generation the NEXT step records into
  int last_f_mb, last_mbs;
  uint8_t *last_b, *last_w;         // [last_mbs]
  int have_step_events;
  hipEvent_t *ev_pool;     // events recorded after B ops, waited on by their W ops
  int ev_pool_size;
  int ev_next;
  // which B units have been issued since the last reset: bitmap over (layer, mb, unit)
  uint8_t *b_done;
  size_t b_done_size;
  int b_layers, b_mbs;
  // events that order the copy stream of the activation offload against its producer / consumer streams
  // (a stream wait refers to the record that precedes it, so the ring may wrap)
  hipEvent_t ev_copy[16];
  int ev_copy_made, ev_copy_next;
  // set by stp_braid_step while it issues a step on distinct streams: kernels launched then share the GPU
  // with the other streams' kernels, which changes the best GEMM tile
  int concurrent;
  // Tile preferences of the bf16 GEMM for launches issued while stp_braid_step runs on concurrent streams
  // (stp_gemm_tile_hint): what is fastest there depends on the kernels of the other streams, which no model of
  // the GEMM alone sees, so a caller may measure and say.
  struct { int32_t M, N, K, layout, tile_m, tile_n; } tile_hint[STP_TILE_HINTS];
  int n_tile_hints;
  // plans of the attention kernels for the shapes seen so far (making one simulates the dispatch)
  stp_attn_plan attn_plan[STP_ATTN_PLAN_CACHE];
  int attn_plan_n, attn_plan_next;
};

static inline int stp_fail(stp_ctx *ctx, int status, const char *fmt, const char *a = "", long b = 0, long c = 0) {
  if (ctx) snprintf(ctx->err, sizeof(ctx->err), fmt, a, b, c);
  return status;
}

#define STP_HIP(ctx, call)                                                                 \
  do {                                                                                     \
    hipError_t e_ = (call);                                                                \
    if (e_ != hipSuccess) {                                                                \
      if (ctx) snprintf((ctx)->err, sizeof((ctx)->err), "%s failed: %s (%s:%d)", #call,    \
                        hipGetErrorString(e_), __FILE__, __LINE__);                        \
      return STP_EHIP;                                                                     \
    }                                                                                      \
  } while (0)

#define STP_LAUNCH_CHECK(ctx) STP_HIP(ctx, hipGetLastError())

static inline bool stp_aligned16(const void *p) { return (((uintptr_t)p) & 15u) == 0; }
static inline size_t stp_align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
static inline size_t stp_elem_size(int dtype) { return dtype == STP_BF16 ? 2 : 4; }

// ---- device-side 8-element vector access, math in fp32 -----------------------------
template <typename T> struct Vec8;
template <> struct Vec8<float> {
  static __device__ __forceinline__ void load(const float *p, float (&v)[8]) {
    float4 a = *reinterpret_cast<const float4 *>(p);
    float4 b = *reinterpret_cast<const float4 *>(p + 4);
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
  }
  static __device__ __forceinline__ void store(float *p, const float (&v)[8]) {
    *reinterpret_cast<float4 *>(p) = make_float4(v[0], v[1], v[2], v[3]);
    *reinterpret_cast<float4 *>(p + 4) = make_float4(v[4], v[5], v[6], v[7]);
  }
};
template <> struct Vec8<bf16_t> {
  static __device__ __forceinline__ void load(const bf16_t *p, float (&v)[8]) {
    uint4 u = *reinterpret_cast<const uint4 *>(p);
    uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
    for (int i = 0; i < 4; i++) {
      v[2 * i] = __uint_as_float(w[i] << 16);
      v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  }
  static __device__ __forceinline__ void store(bf16_t *p, const float (&v)[8]) {
    bf16x8_t o;
#pragma unroll
    for (int i = 0; i < 8; i++) o[i] = (bf16_t)v[i];
    *reinterpret_cast<bf16x8_t *>(p) = o;
  }
};

template <typename T> __device__ __forceinline__ float to_f32(T x) { return (float)x; }
template <typename T> __device__ __forceinline__ T from_f32(float x) { return (T)x; }

// The value lane (l ^ 32) holds, without the LDS round trip of a shuffle: v_permlane32_swap exchanges the
// upper half of one register with the lower half of another.  (Inline assembly: the builtin form was
// seen to return the same register for both results.  The no-ops cover the wait states between a
// vector write and the lane permute, which the compiler cannot insert inside assembly.)
__device__ __forceinline__ float other_half(float v) {
  float a = v, b = v;
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32_e32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
  // a = [v.lo | v.lo], b = [v.hi | v.hi]: lanes below 32 want b, the others a
  return (threadIdx.x & 32) ? a : b;
}

// Sum / maximum over the 64 lanes of a wave, the result in every lane.  Within a row of 16 lanes by cross-lane
// operand modifiers (quad permutes, then the half-row and row mirrors: no LDS round trips as a shuffle has),
// then the four rows through scalar registers, (r0 + r1) + (r2 + r3).
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, false));
}
__device__ __forceinline__ float lane_f32(float v, int lane) {
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), lane));
}
__device__ __forceinline__ float wave_sum(float v) {
  v += dpp_f32<0xB1>(v);    // quad_perm [1,0,3,2]
  v += dpp_f32<0x4E>(v);    // quad_perm [2,3,0,1]
  v += dpp_f32<0x141>(v);   // row_half_mirror
  v += dpp_f32<0x140>(v);   // row_mirror
  return (lane_f32(v, 0) + lane_f32(v, 16)) + (lane_f32(v, 32) + lane_f32(v, 48));
}
__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, dpp_f32<0xB1>(v));
  v = fmaxf(v, dpp_f32<0x4E>(v));
  v = fmaxf(v, dpp_f32<0x141>(v));
  v = fmaxf(v, dpp_f32<0x140>(v));
  return fmaxf(fmaxf(lane_f32(v, 0), lane_f32(v, 16)), fmaxf(lane_f32(v, 32), lane_f32(v, 48)));
}

// exact GELU x*Phi(x) and its derivative Phi(x) + x*phi(x)
__device__ __forceinline__ float gelu_f(float x) { return 0.5f * x * (1.0f + erff(x * 0.70710678118654752f)); }
__device__ __forceinline__ float gelu_grad_f(float x) {
  float Phi = 0.5f * (1.0f + erff(x * 0.70710678118654752f));
  float phi = 0.3989422804014327f * __expf(-0.5f * x * x);
  return Phi + x * phi;
}
// The same two for bf16 storage, where the rounding of the result (2^-9) hides an absolute error of 1e-7: the
// normal distribution function from the rational-times-exponential approximation of erfc (Abramowitz & Stegun
// 7.1.26, |error| < 1.5e-7 in erf), branch-free: 0.5 erfc(|x|/sqrt 2) = 0.5 t (a1 + t (a2 + ... )) exp(-x^2/2),
// t = 1 / (1 + p |x| / sqrt 2); the lower tail is taken directly (no cancellation), the upper as 1 - tail.
// `e` returns exp(-x^2/2), which the derivative needs as well.
__device__ __forceinline__ float normal_cdf_fast(float x, float &e) {
  const float ax = fabsf(x) * 0.70710678118654752f;
  const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, ax, 1.0f));
  float p = fmaf(t, 1.061405429f, -1.453152027f);
  p = fmaf(t, p, 1.421413741f);
  p = fmaf(t, p, -0.284496736f);
  p = fmaf(t, p, 0.254829592f);
  e = __builtin_amdgcn_exp2f(ax * ax * -1.4426950408889634f);
  const float q = 0.5f * p * t * e;
  return x < 0.f ? q : 1.0f - q;
}
template <typename T> __device__ __forceinline__ float gelu_t(float x) {
  if constexpr (sizeof(T) == 4) return gelu_f(x);
  float e;
  return x * normal_cdf_fast(x, e);
}
template <typename T> __device__ __forceinline__ float gelu_grad_t(float x) {
  if constexpr (sizeof(T) == 4) return gelu_grad_f(x);
  float e;
  const float Phi = normal_cdf_fast(x, e);
  return fmaf(x * 0.3989422804014327f, e, Phi);
}
__device__ __forceinline__ float sigmoid_f(float x) { return 1.0f / (1.0f + __expf(-x)); }

// ---- kernel launchers implemented in the .hip files ---------------------------------
int stp_launch_gemm_bf16(stp_ctx *ctx, const stp_gemm_args *a, hipStream_t s);
int stp_launch_gemm_f32(stp_ctx *ctx, const stp_gemm_args *a, hipStream_t s);
int stp_launch_attn_fwd_bf16(stp_ctx *ctx, const stp_layer_desc *d, const void *qkv, void *out, float *lse, float *ws,
                             size_t ws_bytes, hipStream_t s);
int stp_launch_attn_bwd_bf16(stp_ctx *ctx, const stp_layer_desc *d, const void *qkv, const void *out, const float *lse,
                             const void *dout, float *delta, void *dqkv, float *ws, size_t ws_bytes, hipStream_t s);
// grouped-query attention: key / value heads of a rank and the width of its QKV activation
static inline int stp_kv_heads(const stp_layer_desc *d) { return d->kv_heads_local > 0 ? d->kv_heads_local : d->heads_local; }
static inline int stp_qkv_width(const stp_layer_desc *d) { return (d->heads_local + 2 * stp_kv_heads(d)) * d->head_dim; }

// The plan for one attention kernel.  kind: 0 forward, 1 dkv, 2 dq; steps[x] is the number of steps of block
// x; zcount the number of (head, sequence) pairs that repeat the same blocks.  With a context the plan is
// cached there (tag: kind and the layer's attention shape); without one it lives in a thread-local slot.
const stp_attn_plan *stp_attn_plan_get(stp_ctx *ctx, int kind, const stp_layer_desc *d, int nblocks, const int *steps, int zcount);
// the context's (or, without one, the thread's) cache slot for a plan with this tag; *hit says whether it is filled
stp_attn_plan *stp_attn_plan_slot(stp_ctx *ctx, const int key[8], bool *hit);
// the plan's estimate of a workgroup's time in microseconds: `len` steps of a kernel of this kind
double stp_attn_item_cost(int kind, int len);
// the plan of one kernel for a layer shape (kind as above); bf16 shapes only
const stp_attn_plan *stp_attn_plan_for(stp_ctx *ctx, const stp_layer_desc *d, int kind);
const stp_attn_plan *stp_attn_bwd_plan_for(stp_ctx *ctx, const stp_layer_desc *d, int kind);

size_t stp_attn_fwd_ws_bytes(const stp_layer_desc *d);   // workspace the bf16 attention kernels need (chunk partials)
size_t stp_attn_bwd_ws_bytes(const stp_layer_desc *d);
int stp_launch_attn_fwd_generic(stp_ctx *ctx, const stp_layer_desc *d, const void *qkv, void *out, float *lse, hipStream_t s);
int stp_launch_attn_bwd_generic(stp_ctx *ctx, const stp_layer_desc *d, const void *qkv, const void *out, const float *lse,
                                const void *dout, float *delta, void *dqkv, hipStream_t s);
// device address of the fixed scratch array of stp_colsum_noalloc on `device` (the current device); a lookup, no allocation
int stp_noalloc_init(stp_ctx *ctx, int device);
// Launch geometry that also sizes the workspace.  Norm backward: 256-thread row groups that stride over the rows,
// one partial per group.
static inline int stp_norm_bwd_blocks(int rows, int h) {
  (void)h;
  return rows < 512 ? rows : 512;
}
// Column sum: stage-1 patches of STP_COLSUM_ROWS rows, one partial row each
#define STP_COLSUM_ROWS 64
static inline int stp_colsum_slabs(int rows) { return (rows + STP_COLSUM_ROWS - 1) / STP_COLSUM_ROWS; }
// workspace lane: a third of the caller's workspace
static inline char *stp_ws_lane(stp_ctx *ctx, int lane, size_t *bytes) {
  size_t third = (ctx->ws_bytes / 3) & ~(size_t)255;
  *bytes = third;
  return ctx->ws ? ctx->ws + (size_t)lane * third : nullptr;
}

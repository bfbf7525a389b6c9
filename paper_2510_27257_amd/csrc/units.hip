// The C ABI: context, shape checks, stash layout and the F / B / W units composed
// from the kernels (Section 3 of the paper; Eq. 1 for the folded residual in
// forward, Eq. 2 for the "+1" path in backward; B / W split after Zero Bubble).
#include <stdlib.h>
#include <string.h>
#include <new>
#include "common.h"

int stp_launch_rowdot(stp_ctx *ctx, const stp_layer_desc *d, const void *a, const void *b, float *delta, hipStream_t s);

extern "C" const char *stp_status_str(int st) {
  switch (st) {
    case STP_OK: return "STP_OK";
    case STP_EINVAL: return "STP_EINVAL";
    case STP_ESHAPE: return "STP_ESHAPE";
    case STP_EALIGN: return "STP_EALIGN";
    case STP_ENOSPACE: return "STP_ENOSPACE";
    case STP_ESEQ: return "STP_ESEQ";
    case STP_EUNSUPPORTED: return "STP_EUNSUPPORTED";
    case STP_EHIP: return "STP_EHIP";
  }
  return "STP_?";
}

extern "C" int stp_create(stp_ctx **out, int device) {
  if (!out) return STP_EINVAL;
  *out = nullptr;
  int count = 0;
  if (hipGetDeviceCount(&count) != hipSuccess || device < 0 || device >= count) return STP_EHIP;
  if (hipSetDevice(device) != hipSuccess) return STP_EHIP;
  stp_ctx *c = new (std::nothrow) stp_ctx();
  if (!c) return STP_ENOSPACE;
  memset(c, 0, sizeof(*c));
  c->device = device;
  (void)stp_noalloc_init(c, device);   // best effort here; stp_colsum_noalloc repeats the lookup and reports its failure
  c->err[0] = 0;
  *out = c;
  return STP_OK;
}

extern "C" int stp_destroy(stp_ctx *ctx) {
  if (!ctx) return STP_EINVAL;
  if (ctx->have_step_events)
    for (int i = 0; i < 6; i++) (void)hipEventDestroy(ctx->ev_step[i / 3][i % 3]);
  for (int i = 0; i < ctx->ev_pool_size; i++) (void)hipEventDestroy(ctx->ev_pool[i]);
  for (int i = 0; i < ctx->ev_copy_made; i++) (void)hipEventDestroy(ctx->ev_copy[i]);
  free(ctx->ev_pool);
  free(ctx->b_done);
  free(ctx->last_b);   // last_w points into the same block
  delete ctx;
  return STP_OK;
}

extern "C" const char *stp_last_error(const stp_ctx *ctx) { return ctx ? ctx->err : "null context"; }

extern "C" int stp_check_desc(const stp_layer_desc *d) {
  if (!d) return STP_EINVAL;
  if (d->dtype != STP_F32 && d->dtype != STP_BF16) return STP_EINVAL;
  if (d->norm != STP_NORM_LN && d->norm != STP_NORM_RMS) return STP_EINVAL;
  if (d->act != STP_ACT_GELU && d->act != STP_ACT_SWIGLU) return STP_EINVAL;
  if (d->tp < 1 || d->seq < 1 || d->mbsz < 1 || d->heads_local < 1) return STP_ESHAPE;
  if (d->kv_heads_local < 0 || (d->kv_heads_local > 0 && d->heads_local % d->kv_heads_local)) return STP_ESHAPE;
  if (d->hidden < 8 || d->hidden % 8 || d->hidden > 8192) return STP_ESHAPE;
  if (d->ffn_local < 8 || d->ffn_local % 8) return STP_ESHAPE;
  if (d->head_dim < 8 || d->head_dim % 8 || d->head_dim > 128) return STP_ESHAPE;
  if (d->dtype == STP_BF16 && d->head_dim != 64 && d->head_dim != 128) return STP_ESHAPE;
  if (d->rope && d->head_dim % 16) return STP_ESHAPE;
  if (((long)d->seq * d->mbsz) % 8) return STP_ESHAPE;  // the W GEMMs contract over tokens in 16-byte steps
  if ((long)d->seq * d->mbsz > (1L << 24)) return STP_ESHAPE;
  if (!(d->eps > 0.f)) return STP_EINVAL;
  if (d->rope && !(d->rope_base > 1.f)) return STP_EINVAL;
  return STP_OK;
}

static size_t field_bytes(const stp_layer_desc *d, int f) {
  const size_t T = (size_t)d->seq * d->mbsz, es = stp_elem_size(d->dtype);
  const size_t h = d->hidden, a = (size_t)d->heads_local * d->head_dim, ff = d->ffn_local;
  const bool sw = d->act == STP_ACT_SWIGLU;
  switch (f) {
    case STP_ST_X_LN: case STP_ST_Z_LN: case STP_ST_X_ATTN: case STP_ST_DX_ATTN: case STP_ST_DZ: case STP_ST_DX_LN:
      return T * h * es;
    case STP_ST_STATS1: case STP_ST_STATS2: return T * 2 * sizeof(float);
    case STP_ST_QKV: case STP_ST_DQKV: return T * (size_t)stp_qkv_width(d) * es;
    case STP_ST_CTX: case STP_ST_DCTX: return T * a * es;
    case STP_ST_LSE: case STP_ST_DELTA: return (size_t)d->mbsz * d->heads_local * d->seq * sizeof(float);
    case STP_ST_H: case STP_ST_G: case STP_ST_DH: return T * ff * es;
    case STP_ST_HU: case STP_ST_DHU: case STP_ST_DG: return sw ? T * ff * es : 0;
  }
  return 0;
}

extern "C" int stp_stash_field(const stp_layer_desc *d, int field, size_t *offset, size_t *bytes) {
  int rc = stp_check_desc(d);
  if (rc != STP_OK) return rc;
  if (field < 0 || field >= STP_ST_NFIELDS || !offset || !bytes) return STP_EINVAL;
  size_t off = 0;
  for (int f = 0; f < field; f++) off += stp_align_up(field_bytes(d, f), 256);
  *offset = off;
  *bytes = field_bytes(d, field);
  return STP_OK;
}

extern "C" int stp_stash_bytes(const stp_layer_desc *d, size_t *bytes) {
  int rc = stp_check_desc(d);
  if (rc != STP_OK) return rc;
  if (!bytes) return STP_EINVAL;
  size_t off = 0;
  for (int f = 0; f < STP_ST_NFIELDS; f++) off += stp_align_up(field_bytes(d, f), 256);
  *bytes = off;
  return STP_OK;
}

static size_t ws_lane_bytes(const stp_layer_desc *d) {
  const size_t T = (size_t)d->seq * d->mbsz;
  const size_t h = d->hidden, a3 = (size_t)stp_qkv_width(d), ff = d->ffn_local;
  size_t norm = (size_t)stp_norm_bwd_blocks((int)T, (int)h) * 3 * h * sizeof(float);   // [gain | bias | residual sum] per workgroup
  size_t widest = h > a3 ? h : a3;
  if (ff > widest) widest = ff;
  size_t cs = (size_t)stp_colsum_slabs((int)T) * widest * sizeof(float);
  size_t need = norm > cs ? norm : cs;
  if (d->dtype == STP_BF16) {
    size_t af = stp_attn_fwd_ws_bytes(d), ab = stp_attn_bwd_ws_bytes(d);
    if (af > need) need = af;
    if (ab > need) need = ab;
  }
  return stp_align_up(need, 256);
}

extern "C" int stp_workspace_bytes(const stp_layer_desc *d, size_t *bytes) {
  int rc = stp_check_desc(d);
  if (rc != STP_OK) return rc;
  if (!bytes) return STP_EINVAL;
  *bytes = 3 * ws_lane_bytes(d) + 256;
  return STP_OK;
}

extern "C" int stp_attention_plan(const stp_layer_desc *d, int kind, int32_t *chunk_steps, int32_t *max_chunks, int32_t *n_items,
                                  uint16_t *items, size_t items_cap) {
  int rc = stp_check_desc(d);
  if (rc != STP_OK) return rc;
  if (kind < 0 || kind > 2 || !chunk_steps || !max_chunks || !n_items) return STP_EINVAL;
  if (d->dtype != STP_BF16) return STP_EUNSUPPORTED;      // the fp32 attention kernels are not chunked
  const stp_attn_plan *p = stp_attn_plan_for(nullptr, d, kind);
  *chunk_steps = p->chunk_steps;
  *max_chunks = p->max_chunks;
  *n_items = p->n_items;
  if (items) {
    if (items_cap < (size_t)p->n_items) return STP_ENOSPACE;
    for (int i = 0; i < p->n_items; i++) items[i] = p->order.item[i];
  }
  return STP_OK;
}

extern "C" int stp_set_workspace(stp_ctx *ctx, void *p, size_t bytes) {
  if (!ctx) return STP_EINVAL;
  if (p && !stp_aligned16(p)) return stp_fail(ctx, STP_EALIGN, "stp_set_workspace: pointer must be 16-byte aligned%s");
  ctx->ws = (char *)p;
  ctx->ws_bytes = p ? bytes : 0;
  return STP_OK;
}

// ---------------------------------------------------------------------------
extern "C" int stp_gemm_tile_hint(stp_ctx *ctx, int32_t M, int32_t N, int32_t K, int a_trans, int b_trans, int32_t tile_m,
                                  int32_t tile_n) {
  if (!ctx) return STP_EINVAL;
  const int layout = 2 * (a_trans ? 0 : 1) + (b_trans ? 1 : 0);
  int at = -1;
  for (int i = 0; i < ctx->n_tile_hints; i++) {
    const auto &h = ctx->tile_hint[i];
    if (h.M == M && h.N == N && h.K == K && h.layout == layout) { at = i; break; }
  }
  if (tile_m == 0 && tile_n == 0) {          // forget the preference
    if (at >= 0) ctx->tile_hint[at] = ctx->tile_hint[--ctx->n_tile_hints];
    return STP_OK;
  }
  const bool square = (tile_m == 128 || tile_m == 256) && (tile_n == 128 || tile_n == 256);
  const bool wide = tile_m == 192 && tile_n == 256 && !a_trans;
  if (!square && !wide) return stp_fail(ctx, STP_EINVAL, "stp_gemm_tile_hint: the tile must be 128 or 256 each way, or 192 x 256 with a_trans = 0%s");
  if (M <= 0 || N <= 0 || K <= 0) return stp_fail(ctx, STP_ESHAPE, "stp_gemm_tile_hint: bad shape%s");
  if (at < 0) {
    if (ctx->n_tile_hints >= STP_TILE_HINTS) return stp_fail(ctx, STP_ENOSPACE, "stp_gemm_tile_hint: table full%s");
    at = ctx->n_tile_hints++;
  }
  ctx->tile_hint[at] = {M, N, K, layout, tile_m, tile_n};
  return STP_OK;
}

extern "C" int stp_gemm_tile_hints_clear(stp_ctx *ctx) {
  if (!ctx) return STP_EINVAL;
  ctx->n_tile_hints = 0;
  return STP_OK;
}

extern "C" int stp_gemm(stp_ctx *ctx, const stp_gemm_args *g, void *hip_stream) {
  if (!ctx) return STP_EINVAL;
  if (!g || !g->A || !g->B || !g->C) return stp_fail(ctx, STP_EINVAL, "stp_gemm: null pointer%s");
  if (g->dtype != STP_BF16 && g->dtype != STP_F32) return stp_fail(ctx, STP_EINVAL, "stp_gemm: bad dtype%s");
  if (g->M < 0 || g->N < 0 || g->K < 0) return stp_fail(ctx, STP_ESHAPE, "stp_gemm: negative dimension%s");
  if (g->M % 8 || g->N % 8 || g->K % 8 || g->lda % 8 || g->ldb % 8 || g->ldc % 8)
    return stp_fail(ctx, STP_ESHAPE, "stp_gemm: M, N, K and leading dimensions must be multiples of 8%s");
  if (g->lda < (g->a_trans ? g->M : g->K) || g->ldb < (g->b_trans ? g->K : g->N) || g->ldc < g->N)
    return stp_fail(ctx, STP_ESHAPE, "stp_gemm: leading dimension smaller than the row length%s");
  if (!stp_aligned16(g->A) || !stp_aligned16(g->B) || !stp_aligned16(g->C) || (g->bias && !stp_aligned16(g->bias)) ||
      (g->resid && !stp_aligned16(g->resid)))
    return stp_fail(ctx, STP_EALIGN, "stp_gemm: pointers must be 16-byte aligned%s");
  if (g->resid && (g->ldr % 8 || g->ldr < g->N)) return stp_fail(ctx, STP_ESHAPE, "stp_gemm: bad ldr%s");
  if (g->epilogue < 0 || g->epilogue > 2) return stp_fail(ctx, STP_EINVAL, "stp_gemm: bad epilogue%s");
  if (g->epilogue == 1 && (!g->C2 || g->ld2 < g->N)) return stp_fail(ctx, STP_EINVAL, "stp_gemm: epilogue 1 needs C2/ld2%s");
  if (g->epilogue == 2 && (!g->aux || g->ld2 < g->N)) return stp_fail(ctx, STP_EINVAL, "stp_gemm: epilogue 2 needs aux/ld2%s");
  if (g->epilogue && g->c_f32_accum) return stp_fail(ctx, STP_EINVAL, "stp_gemm: epilogue with fp32 accumulation%s");
  if (g->tile_m || g->tile_n) {
    const bool square = (g->tile_m == 128 || g->tile_m == 256) && (g->tile_n == 128 || g->tile_n == 256);
    const bool wide = g->tile_m == 192 && g->tile_n == 256 && !g->a_trans;      // needs a k-contiguous A
    const bool ok = (square || wide) && g->dtype == STP_BF16 && g->K % 32 == 0;
    if (!ok)
      return stp_fail(ctx, STP_EINVAL, "stp_gemm: tile_m / tile_n must both be 0, or 128 or 256 each, or 192 x 256 with a_trans = 0, "
                                       "for bf16 with K %% 32 == 0%s");
  }
  if (g->M == 0 || g->N == 0) return STP_OK;
  hipStream_t s = (hipStream_t)hip_stream;
  return g->dtype == STP_BF16 ? stp_launch_gemm_bf16(ctx, g, s) : stp_launch_gemm_f32(ctx, g, s);
}

static int attn_args_ok(stp_ctx *ctx, const stp_layer_desc *d, const char *who) {
  int rc = stp_check_desc(d);
  if (rc != STP_OK) return stp_fail(ctx, rc, "%s: layer description rejected", who);
  return STP_OK;
}

extern "C" int stp_attention_forward(stp_ctx *ctx, const stp_layer_desc *d, const void *qkv, void *out, float *lse,
                                     int lane, void *hip_stream) {
  if (!ctx) return STP_EINVAL;
  if (!d || !qkv || !out || !lse) return stp_fail(ctx, STP_EINVAL, "stp_attention_forward: null pointer%s");
  int rc = attn_args_ok(ctx, d, "stp_attention_forward");
  if (rc != STP_OK) return rc;
  if (!stp_aligned16(qkv) || !stp_aligned16(out)) return stp_fail(ctx, STP_EALIGN, "stp_attention_forward: alignment%s");
  if (lane < 0 || lane > 2) return stp_fail(ctx, STP_EINVAL, "stp_attention_forward: lane must be 0..2%s");
  hipStream_t s = (hipStream_t)hip_stream;
  if (d->dtype == STP_BF16) {
    size_t lane_bytes;
    char *ws = stp_ws_lane(ctx, lane, &lane_bytes);
    return stp_launch_attn_fwd_bf16(ctx, d, qkv, out, lse, (float *)ws, lane_bytes, s);
  }
  return stp_launch_attn_fwd_generic(ctx, d, qkv, out, lse, s);
}

extern "C" int stp_attention_backward(stp_ctx *ctx, const stp_layer_desc *d, const void *qkv, const void *out,
                                      const float *lse, const void *dout, float *delta, void *dqkv, int lane,
                                      void *hip_stream) {
  if (!ctx) return STP_EINVAL;
  if (!d || !qkv || !out || !lse || !dout || !delta || !dqkv)
    return stp_fail(ctx, STP_EINVAL, "stp_attention_backward: null pointer%s");
  int rc = attn_args_ok(ctx, d, "stp_attention_backward");
  if (rc != STP_OK) return rc;
  if (!stp_aligned16(qkv) || !stp_aligned16(out) || !stp_aligned16(dout) || !stp_aligned16(dqkv))
    return stp_fail(ctx, STP_EALIGN, "stp_attention_backward: alignment%s");
  if (lane < 0 || lane > 2) return stp_fail(ctx, STP_EINVAL, "stp_attention_backward: lane must be 0..2%s");
  hipStream_t s = (hipStream_t)hip_stream;
  if (d->dtype == STP_BF16) {
    size_t lane_bytes;
    char *ws = stp_ws_lane(ctx, lane, &lane_bytes);
    return stp_launch_attn_bwd_bf16(ctx, d, qkv, out, lse, dout, delta, dqkv, (float *)ws, lane_bytes, s);
  }
  return stp_launch_attn_bwd_generic(ctx, d, qkv, out, lse, dout, delta, dqkv, s);
}

// ---------------------------------------------------------------------------
// unit composition
// ---------------------------------------------------------------------------
struct Fields {
  char *p[STP_ST_NFIELDS];
};

static int resolve_stash(stp_ctx *ctx, const stp_layer_desc *d, const stp_stash *st, Fields *f) {
  if (!st || !st->base) return stp_fail(ctx, STP_EINVAL, "stash is null%s");
  if (!stp_aligned16(st->base)) return stp_fail(ctx, STP_EALIGN, "stash must be 16-byte aligned%s");
  size_t need = 0;
  stp_stash_bytes(d, &need);
  if (st->bytes < need) return stp_fail(ctx, STP_ENOSPACE, "stash too small%s: need %ld bytes, have %ld", "", (long)need, (long)st->bytes);
  size_t off = 0;
  for (int i = 0; i < STP_ST_NFIELDS; i++) {
    f->p[i] = (char *)st->base + off;
    off += stp_align_up(field_bytes(d, i), 256);
  }
  return STP_OK;
}

static stp_gemm_args gemm_base(const stp_layer_desc *d, int M, int N, int K) {
  stp_gemm_args g;
  memset(&g, 0, sizeof(g));
  g.dtype = d->dtype; g.M = M; g.N = N; g.K = K;
  g.bias_scale = 1.f; g.resid_scale = 1.f;
  return g;
}

#define RET_IF(x) do { int rc_ = (x); if (rc_ != STP_OK) return rc_; } while (0)

static int common_checks(stp_ctx *ctx, const stp_layer_desc *d, int unit, int lane, const char *who) {
  if (!d) return stp_fail(ctx, STP_EINVAL, "%s: null layer description", who);
  int rc = stp_check_desc(d);
  if (rc != STP_OK) return stp_fail(ctx, rc, "%s: layer description rejected", who);
  if (unit < STP_PRE_ATTN || unit > STP_MLP) return stp_fail(ctx, STP_EINVAL, "%s: bad unit", who);
  if (lane < 0 || lane > 2) return stp_fail(ctx, STP_EINVAL, "%s: lane must be 0..2", who);
  return STP_OK;
}

static int need_ptr(stp_ctx *ctx, const void *p, const char *what) {
  if (!p) return stp_fail(ctx, STP_EINVAL, "missing argument: %s", what);
  if (!stp_aligned16(p)) return stp_fail(ctx, STP_EALIGN, "argument not 16-byte aligned: %s", what);
  return STP_OK;
}

extern "C" int stp_forward_unit(stp_ctx *ctx, const stp_layer_desc *d, int unit, const stp_weights *w, const void *x_in,
                                const void *x_resid, void *y_out, const stp_stash *stash, int lane, void *hip_stream) {
  if (!ctx) return STP_EINVAL;
  RET_IF(common_checks(ctx, d, unit, lane, "stp_forward_unit"));
  if (!w) return stp_fail(ctx, STP_EINVAL, "stp_forward_unit: null weights%s");
  Fields f;
  RET_IF(resolve_stash(ctx, d, stash, &f));
  const int T = d->seq * d->mbsz, h = d->hidden, a = d->heads_local * d->head_dim, ff = d->ffn_local;
  const float inv_t = 1.0f / (float)d->tp;
  const bool bias = d->has_bias != 0;
  switch (unit) {
    case STP_PRE_ATTN:
    case STP_PRE_MLP: {
      const bool first = unit == STP_PRE_ATTN;
      const void *g = first ? w->norm1_g : w->norm2_g, *b = first ? w->norm1_b : w->norm2_b;
      RET_IF(need_ptr(ctx, x_in, "x_in"));
      RET_IF(need_ptr(ctx, g, "norm gain"));
      return stp_norm_forward(ctx, d->dtype, d->norm, T, h, d->eps, x_in, g, d->norm == STP_NORM_LN ? b : nullptr,
                              f.p[first ? STP_ST_X_LN : STP_ST_Z_LN], (float *)f.p[first ? STP_ST_STATS1 : STP_ST_STATS2],
                              hip_stream);
    }
    case STP_ATTN: {
      RET_IF(need_ptr(ctx, x_resid, "x_resid"));
      RET_IF(need_ptr(ctx, y_out, "y_out"));
      RET_IF(need_ptr(ctx, w->w_qkv, "w_qkv"));
      RET_IF(need_ptr(ctx, w->w_o, "w_o"));
      if (bias) { RET_IF(need_ptr(ctx, w->b_qkv, "b_qkv")); RET_IF(need_ptr(ctx, w->b_o, "b_o")); }
      stp_gemm_args g = gemm_base(d, T, stp_qkv_width(d), h);
      g.A = f.p[STP_ST_X_LN]; g.lda = h;
      g.B = w->w_qkv; g.ldb = stp_qkv_width(d);
      g.C = f.p[STP_ST_QKV]; g.ldc = stp_qkv_width(d);
      g.bias = bias ? w->b_qkv : nullptr;
      RET_IF(stp_gemm(ctx, &g, hip_stream));
      if (d->rope) RET_IF(stp_rope(ctx, d, f.p[STP_ST_QKV], 0, hip_stream));
      RET_IF(stp_attention_forward(ctx, d, f.p[STP_ST_QKV], f.p[STP_ST_CTX], (float *)f.p[STP_ST_LSE], lane, hip_stream));
      g = gemm_base(d, T, h, a);
      g.A = f.p[STP_ST_CTX]; g.lda = a;
      g.B = w->w_o; g.ldb = h;
      g.C = y_out; g.ldc = h;
      g.bias = bias ? w->b_o : nullptr; g.bias_scale = inv_t;        // Eq. 1: every rank adds 1/t of the shared terms
      g.resid = x_resid; g.ldr = h; g.resid_scale = inv_t;           //        detach(X)/t
      return stp_gemm(ctx, &g, hip_stream);
    }
    case STP_MLP: {
      RET_IF(need_ptr(ctx, x_resid, "x_resid"));
      RET_IF(need_ptr(ctx, y_out, "y_out"));
      RET_IF(need_ptr(ctx, w->w_fc1, "w_fc1"));
      RET_IF(need_ptr(ctx, w->w_fc2, "w_fc2"));
      if (bias) { RET_IF(need_ptr(ctx, w->b_fc1, "b_fc1")); RET_IF(need_ptr(ctx, w->b_fc2, "b_fc2")); }
      stp_gemm_args g = gemm_base(d, T, ff, h);
      g.A = f.p[STP_ST_Z_LN]; g.lda = h;
      g.B = w->w_fc1; g.ldb = ff;
      g.C = f.p[STP_ST_H]; g.ldc = ff;
      g.bias = bias ? w->b_fc1 : nullptr;
      if (d->act == STP_ACT_GELU) {
        g.epilogue = 1; g.C2 = f.p[STP_ST_G]; g.ld2 = ff;
        RET_IF(stp_gemm(ctx, &g, hip_stream));
      } else {
        RET_IF(need_ptr(ctx, w->w_up, "w_up"));
        RET_IF(stp_gemm(ctx, &g, hip_stream));
        g.B = w->w_up; g.C = f.p[STP_ST_HU]; g.bias = nullptr;
        RET_IF(stp_gemm(ctx, &g, hip_stream));
        RET_IF(stp_swiglu_forward(ctx, d->dtype, (size_t)T * ff, f.p[STP_ST_H], f.p[STP_ST_HU], f.p[STP_ST_G], hip_stream));
      }
      g = gemm_base(d, T, h, ff);
      g.A = f.p[STP_ST_G]; g.lda = ff;
      g.B = w->w_fc2; g.ldb = h;
      g.C = y_out; g.ldc = h;
      g.bias = bias ? w->b_fc2 : nullptr; g.bias_scale = inv_t;
      g.resid = x_resid; g.ldr = h; g.resid_scale = inv_t;
      return stp_gemm(ctx, &g, hip_stream);
    }
  }
  return STP_EINVAL;
}

extern "C" int stp_backward_input_unit(stp_ctx *ctx, const stp_layer_desc *d, int unit, const stp_weights *w,
                                       const stp_stash *stash, const void *x_in, const void *dy, const void *d_resid,
                                       void *dx, stp_wgrads *wg, int lane, void *hip_stream) {
  if (!ctx) return STP_EINVAL;
  RET_IF(common_checks(ctx, d, unit, lane, "stp_backward_input_unit"));
  if (!w) return stp_fail(ctx, STP_EINVAL, "stp_backward_input_unit: null weights%s");
  Fields f;
  RET_IF(resolve_stash(ctx, d, stash, &f));
  RET_IF(need_ptr(ctx, dy, "dy"));
  RET_IF(need_ptr(ctx, dx, "dx"));
  const int T = d->seq * d->mbsz, h = d->hidden, a = d->heads_local * d->head_dim, ff = d->ffn_local;
  switch (unit) {
    case STP_MLP: {
      RET_IF(need_ptr(ctx, w->w_fc1, "w_fc1"));
      RET_IF(need_ptr(ctx, w->w_fc2, "w_fc2"));
      // dG = dY W2^T ; W2 is [f, h]: as B operand it is [N=f][K=h], contraction contiguous
      stp_gemm_args g = gemm_base(d, T, ff, h);
      g.A = dy; g.lda = h;
      g.B = w->w_fc2; g.ldb = h; g.b_trans = 1;
      if (d->act == STP_ACT_GELU) {
        g.C = f.p[STP_ST_DH]; g.ldc = ff;
        g.epilogue = 2; g.aux = f.p[STP_ST_H]; g.ld2 = ff;            // dH = dG * GELU'(H)
        RET_IF(stp_gemm(ctx, &g, hip_stream));
      } else {
        RET_IF(need_ptr(ctx, w->w_up, "w_up"));
        g.C = f.p[STP_ST_DG]; g.ldc = ff;
        RET_IF(stp_gemm(ctx, &g, hip_stream));
        RET_IF(stp_swiglu_backward(ctx, d->dtype, (size_t)T * ff, f.p[STP_ST_H], f.p[STP_ST_HU], f.p[STP_ST_DG],
                                   f.p[STP_ST_DH], f.p[STP_ST_DHU], hip_stream));
      }
      g = gemm_base(d, T, h, ff);
      g.A = f.p[STP_ST_DH]; g.lda = ff;
      g.B = w->w_fc1; g.ldb = ff; g.b_trans = 1;
      g.C = dx; g.ldc = h;
      RET_IF(stp_gemm(ctx, &g, hip_stream));
      if (d->act == STP_ACT_SWIGLU) {
        g.A = f.p[STP_ST_DHU]; g.B = w->w_up;
        g.resid = dx; g.ldr = h; g.resid_scale = 1.f;                 // dx += dHu Wu^T (same thread reads then writes)
        RET_IF(stp_gemm(ctx, &g, hip_stream));
      }
      return STP_OK;
    }
    case STP_PRE_MLP:
    case STP_PRE_ATTN: {
      const bool first = unit == STP_PRE_ATTN;
      RET_IF(need_ptr(ctx, x_in, "x_in"));
      RET_IF(need_ptr(ctx, d_resid, "d_resid"));
      const void *gam = first ? w->norm1_g : w->norm2_g;
      RET_IF(need_ptr(ctx, gam, "norm gain"));
      float *dgam = wg ? (first ? wg->norm1_g : wg->norm2_g) : nullptr;
      float *dbet = wg ? (first ? wg->norm1_b : wg->norm2_b) : nullptr;
      // The gradient on the residual path is the upstream gradient of the Attn (Pre-Attn-B) / MLP (Pre-MLP-B)
      // unit, so (1/t) of its column sum is the gradient of that unit's row-parallel bias b_o / b_fc2 (Eq. 1
      // adds b/t on every rank).  This unit reads it anyway: it fills the accumulator when it is handed one.
      float *dbias = (wg && d->has_bias) ? (first ? wg->b_o : wg->b_fc2) : nullptr;
      // Eq. 2: dX = norm_bwd(reduced gradient) + 1 * (gradient arriving on the residual path)
      return stp_norm_backward(ctx, d->dtype, d->norm, T, h, x_in, gam, (const float *)f.p[first ? STP_ST_STATS1 : STP_ST_STATS2],
                               dy, d_resid, dx, dgam, dbet, dbias, 1.0f / (float)d->tp, lane, hip_stream);
    }
    case STP_ATTN: {
      RET_IF(need_ptr(ctx, w->w_qkv, "w_qkv"));
      RET_IF(need_ptr(ctx, w->w_o, "w_o"));
      stp_gemm_args g = gemm_base(d, T, a, h);
      g.A = dy; g.lda = h;
      g.B = w->w_o; g.ldb = h; g.b_trans = 1;
      g.C = f.p[STP_ST_DCTX]; g.ldc = a;
      RET_IF(stp_gemm(ctx, &g, hip_stream));
      RET_IF(stp_attention_backward(ctx, d, f.p[STP_ST_QKV], f.p[STP_ST_CTX], (const float *)f.p[STP_ST_LSE],
                                    f.p[STP_ST_DCTX], (float *)f.p[STP_ST_DELTA], f.p[STP_ST_DQKV], lane, hip_stream));
      if (d->rope) RET_IF(stp_rope(ctx, d, f.p[STP_ST_DQKV], 1, hip_stream));
      g = gemm_base(d, T, h, stp_qkv_width(d));
      g.A = f.p[STP_ST_DQKV]; g.lda = stp_qkv_width(d);
      g.B = w->w_qkv; g.ldb = stp_qkv_width(d); g.b_trans = 1;
      g.C = dx; g.ldc = h;
      return stp_gemm(ctx, &g, hip_stream);
    }
  }
  return STP_EINVAL;
}

extern "C" int stp_backward_weight_unit(stp_ctx *ctx, const stp_layer_desc *d, int unit, const stp_stash *stash,
                                        const void *dy, stp_wgrads *wg, int lane, void *hip_stream) {
  if (!ctx) return STP_EINVAL;
  RET_IF(common_checks(ctx, d, unit, lane, "stp_backward_weight_unit"));
  if (unit != STP_ATTN && unit != STP_MLP)
    return stp_fail(ctx, STP_EINVAL, "stp_backward_weight_unit: only the Attn and MLP units have a W part%s");
  if (!wg) return stp_fail(ctx, STP_EINVAL, "stp_backward_weight_unit: null gradient table%s");
  Fields f;
  RET_IF(resolve_stash(ctx, d, stash, &f));
  RET_IF(need_ptr(ctx, dy, "dy"));
  const int T = d->seq * d->mbsz, h = d->hidden, a = d->heads_local * d->head_dim, ff = d->ffn_local;
  const float inv_t = 1.0f / (float)d->tp;
  // dW[in, out] += act^T grad: both operands are [tokens, features], contraction over tokens
  auto wgemm = [&](const void *act, int in, const void *grad, int out, float *dw) -> int {
    if (!dw) return STP_OK;
    stp_gemm_args g = gemm_base(d, in, out, T);
    g.A = act; g.lda = in; g.a_trans = 1;
    g.B = grad; g.ldb = out; g.b_trans = 0;
    g.C = dw; g.ldc = out; g.c_f32_accum = 1;
    return stp_gemm(ctx, &g, hip_stream);
  };
  if (unit == STP_MLP) {
    RET_IF(wgemm(f.p[STP_ST_G], ff, dy, h, wg->w_fc2));
    RET_IF(wgemm(f.p[STP_ST_Z_LN], h, f.p[STP_ST_DH], ff, wg->w_fc1));
    if (d->act == STP_ACT_SWIGLU) RET_IF(wgemm(f.p[STP_ST_Z_LN], h, f.p[STP_ST_DHU], ff, wg->w_up));
    if (d->has_bias) {
      if (wg->b_fc1) RET_IF(stp_colsum(ctx, d->dtype, T, ff, f.p[STP_ST_DH], 1.0f, wg->b_fc1, lane, hip_stream));
      if (wg->b_fc2) RET_IF(stp_colsum(ctx, d->dtype, T, h, dy, inv_t, wg->b_fc2, lane, hip_stream));
    }
    return STP_OK;
  }
  RET_IF(wgemm(f.p[STP_ST_CTX], a, dy, h, wg->w_o));
  RET_IF(wgemm(f.p[STP_ST_X_LN], h, f.p[STP_ST_DQKV], stp_qkv_width(d), wg->w_qkv));
  if (d->has_bias) {
    if (wg->b_qkv) RET_IF(stp_colsum(ctx, d->dtype, T, stp_qkv_width(d), f.p[STP_ST_DQKV], 1.0f, wg->b_qkv, lane, hip_stream));
    if (wg->b_o) RET_IF(stp_colsum(ctx, d->dtype, T, h, dy, inv_t, wg->b_o, lane, hip_stream));
  }
  return STP_OK;
}

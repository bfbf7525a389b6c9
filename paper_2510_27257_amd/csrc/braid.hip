// The braided execution block (Section 3, Fig. 3; Section 4.1 pattern (2); Appendix A):
// the F units of microbatch i are issued on one HIP stream, the B units of an earlier
// microbatch j on a second, the W units on a third, in the caller's interleaved order.
// Only true data dependences are turned into events: a W waits for its B; a stream of a step waits for
// the streams of the previous step whose results it reads or overwrites, and every stream waits for
// the whole of the step before that, so at most two blocks are in flight and a block's tail overlaps
// the head of the next.  The four TP All-Reduce points per layer
// are reported to the caller's boundary callback (no collective runs here).
#include <stdlib.h>
#include <string.h>
#include "common.h"

namespace {

struct Cursor { int layer, unit; bool set; };

inline bool is_first_of_chain(const stp_stage *st, int layer) {
  return layer == 0 || (st->chain_break && st->chain_break[layer]);
}
inline bool is_last_of_chain(const stp_stage *st, int layer) {
  return layer == st->n_layers - 1 || (st->chain_break && st->chain_break[layer + 1]);
}

// next unit in forward order after (layer, unit); false if the chain ends there
inline bool fwd_successor(const stp_stage *st, int layer, int unit, int *nl, int *nu) {
  if (unit < STP_MLP) { *nl = layer; *nu = unit + 1; return true; }
  if (is_last_of_chain(st, layer)) return false;
  *nl = layer + 1; *nu = STP_PRE_ATTN;
  return true;
}
inline bool bwd_successor(const stp_stage *st, int layer, int unit, int *nl, int *nu) {
  if (unit > STP_PRE_ATTN) { *nl = layer; *nu = unit - 1; return true; }
  if (is_first_of_chain(st, layer)) return false;
  *nl = layer - 1; *nu = STP_MLP;
  return true;
}

int validate(const stp_stage *st, const stp_op *ops, size_t n, const uint8_t *b_done, size_t *bad) {
  size_t dummy;
  if (!bad) bad = &dummy;
  *bad = 0;
  if (!st || (!ops && n)) return STP_EINVAL;
  if (st->n_layers < 1 || st->n_microbatches < 1 || !st->desc) return STP_EINVAL;
  const int L = st->n_layers, MB = st->n_microbatches;
  // a layer's output is written straight into the next layer's input slot (and the gradient the other way):
  // the two descriptions must agree on the extent and type of that slot unless a chain break separates them
  for (int l = 0; l + 1 < L; l++) {
    if (st->chain_break && st->chain_break[l + 1]) continue;
    const stp_layer_desc &a = st->desc[l], &b = st->desc[l + 1];
    if ((long)a.seq * a.mbsz != (long)b.seq * b.mbsz || a.hidden != b.hidden || a.dtype != b.dtype) return STP_ESHAPE;
  }
  int f_mb = -1;
  Cursor fcur = {0, 0, false};
  Cursor *bcur = (Cursor *)calloc(MB, sizeof(Cursor));
  uint8_t *b_here = (uint8_t *)calloc((size_t)L * MB * 2, 1);
  if (!bcur || !b_here) { free(bcur); free(b_here); return STP_ENOSPACE; }
  int rc = STP_OK;
  // first pass: the forward microbatch
  for (size_t i = 0; i < n; i++)
    if (ops[i].kind == STP_OP_F) { f_mb = ops[i].microbatch; break; }
  for (size_t i = 0; i < n && rc == STP_OK; i++) {
    const stp_op &o = ops[i];
    *bad = i;
    if (o.kind < STP_OP_F || o.kind > STP_OP_BW || o.unit < STP_PRE_ATTN || o.unit > STP_MLP || o.layer < 0 ||
        o.layer >= L || o.microbatch < 0 || o.microbatch >= MB) { rc = STP_EINVAL; break; }
    if (o.kind == STP_OP_F) {
      if (o.microbatch != f_mb) { rc = STP_ESEQ; break; }         // one forward microbatch per block
      if (fcur.set) {
        int nl, nu;
        bool more = fwd_successor(st, fcur.layer, fcur.unit, &nl, &nu);
        bool chain_start = o.unit == STP_PRE_ATTN && is_first_of_chain(st, o.layer) && !more;
        if (!((more && nl == o.layer && nu == o.unit) || chain_start)) { rc = STP_ESEQ; break; }
      }
      fcur = {o.layer, o.unit, true};
      continue;
    }
    // backward-side op: its microbatch must precede the forward one (Appendix A)
    if (f_mb >= 0 && o.microbatch >= f_mb) { rc = STP_ESEQ; break; }
    const bool has_w = o.unit == STP_ATTN || o.unit == STP_MLP;
    const size_t slot = ((size_t)o.layer * MB + o.microbatch) * 2 + (o.unit == STP_MLP ? 1 : 0);
    if (o.kind == STP_OP_W) {
      if (!has_w) { rc = STP_ESEQ; break; }
      if (!b_here[slot] && !(b_done && b_done[slot])) { rc = STP_ESEQ; break; }  // W needs its B first
      continue;
    }
    Cursor &c = bcur[o.microbatch];
    if (c.set) {
      int nl, nu;
      bool more = bwd_successor(st, c.layer, c.unit, &nl, &nu);
      bool chain_start = o.unit == STP_MLP && is_last_of_chain(st, o.layer) && !more;
      if (!((more && nl == o.layer && nu == o.unit) || chain_start)) { rc = STP_ESEQ; break; }
    }
    c = {o.layer, o.unit, true};
    if (has_w) b_here[slot] = 1;
  }
  if (rc == STP_OK) *bad = n;
  free(bcur);
  free(b_here);
  return rc;
}

int ensure_events(stp_ctx *ctx, int want) {
  if (!ctx->have_step_events) {
    for (int i = 0; i < 6; i++) STP_HIP(ctx, hipEventCreateWithFlags(&ctx->ev_step[i / 3][i % 3], hipEventDisableTiming));
    ctx->have_step_events = 1;
  }
  if (ctx->ev_pool_size < want) {
    hipEvent_t *np = (hipEvent_t *)realloc(ctx->ev_pool, sizeof(hipEvent_t) * want);
    if (!np) return stp_fail(ctx, STP_ENOSPACE, "out of host memory%s");
    ctx->ev_pool = np;
    for (int i = ctx->ev_pool_size; i < want; i++) {
      STP_HIP(ctx, hipEventCreateWithFlags(&ctx->ev_pool[i], hipEventDisableTiming));
      ctx->ev_pool_size = i + 1;
    }
  }
  return STP_OK;
}

}  // namespace

extern "C" int stp_validate_ops(const stp_stage *stage, const stp_op *ops, size_t n_ops, size_t *bad_index) {
  // without a context nothing is known about earlier steps: accept a W whose B is not in the list
  if (!stage || stage->n_layers < 1 || stage->n_microbatches < 1) return STP_EINVAL;
  size_t sz = (size_t)stage->n_layers * stage->n_microbatches * 2;
  uint8_t *all = (uint8_t *)malloc(sz);
  if (!all) return STP_ENOSPACE;
  memset(all, 1, sz);
  int rc = validate(stage, ops, n_ops, all, bad_index);
  free(all);
  return rc;
}

extern "C" int stp_braid_reset(stp_ctx *ctx) {
  if (!ctx) return STP_EINVAL;
  if (ctx->b_done) memset(ctx->b_done, 0, ctx->b_done_size);
  return STP_OK;
}

extern "C" int stp_braid_detach(stp_ctx *ctx) {
  if (!ctx) return STP_EINVAL;
  ctx->ev_next = 0;
  ctx->ev_valid[0] = ctx->ev_valid[1] = 0;
  return STP_OK;
}

extern "C" int stp_braid_step(stp_ctx *ctx, const stp_stage *st, const stp_op *ops, size_t n_ops, void *s_fwd,
                              void *s_bwd, void *s_wgrad, stp_boundary_fn cb, void *user) {
  if (!ctx) return STP_EINVAL;
  if (!st || !st->desc || !st->w || !st->g || !st->stash || !st->act || !st->grad)
    return stp_fail(ctx, STP_EINVAL, "stp_braid_step: null stage table%s");
  if (st->n_layers < 1 || st->n_microbatches < 1) return stp_fail(ctx, STP_EINVAL, "stp_braid_step: empty stage%s");
  const int L = st->n_layers, MB = st->n_microbatches;
  const size_t bsz = (size_t)L * MB * 2;
  if (!ctx->b_done || ctx->b_layers != L || ctx->b_mbs != MB) {
    free(ctx->b_done);
    ctx->b_done = (uint8_t *)calloc(bsz, 1);
    if (!ctx->b_done) return stp_fail(ctx, STP_ENOSPACE, "out of host memory%s");
    ctx->b_done_size = bsz; ctx->b_layers = L; ctx->b_mbs = MB;
  }
  size_t bad = 0;
  int rc = validate(st, ops, n_ops, ctx->b_done, &bad);
  if (rc != STP_OK) return stp_fail(ctx, rc, "stp_braid_step: op list rejected%s at index %ld", "", (long)bad);
  for (int l = 0; l < L; l++) {
    rc = stp_check_desc(&st->desc[l]);
    if (rc != STP_OK) return stp_fail(ctx, rc, "stp_braid_step: layer description rejected%s (layer %ld)", "", (long)l);
  }
  if (n_ops == 0) return STP_OK;
  // every host-side condition of the whole list is checked before the first launch: a step is issued whole or not at all
  for (size_t i = 0; i < n_ops; i++) {
    const stp_op &o = ops[i];
    if (!st->stash[(size_t)o.layer * MB + o.microbatch].base)
      return stp_fail(ctx, STP_EINVAL, "stp_braid_step: null stash%s (op %ld)", "", (long)i);
    const bool tail = o.layer + 1 < L && st->chain_break && st->chain_break[o.layer + 1];
    if (tail && (!st->tail_act || !st->tail_grad))
      return stp_fail(ctx, STP_EINVAL, "stp_braid_step: chain break without tail slots%s (op %ld)", "", (long)i);
  }

  hipStream_t sF = (hipStream_t)s_fwd, sB = (hipStream_t)s_bwd, sW = (hipStream_t)s_wgrad;
  const bool serial = (sF == sB) && (sB == sW);
  hipStream_t streams[3] = {sF, sB, sW};
  // Recording braid steps into a HIP graph is not supported (see stp.h): refuse a capturing stream with a status.
  for (int i = 0; i < 3; i++) {
    hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(streams[i], &cs) != hipSuccess) {
      (void)hipGetLastError();
      return stp_fail(ctx, STP_EHIP, "stp_braid_step: hipStreamIsCapturing failed%s");
    }
    if (cs != hipStreamCaptureStatusNone)
      return stp_fail(ctx, STP_EUNSUPPORTED, "stp_braid_step: a stream is being captured into a HIP graph; that is not supported%s");
  }
  rc = ensure_events(ctx, (int)n_ops);
  if (rc != STP_OK) return rc;
  // What this step touches: its forward microbatch and the microbatches with B / W work.
  int f_mb = -1;
  uint8_t *cur_b = (uint8_t *)calloc(2 * (size_t)MB, 1), *cur_w = cur_b ? cur_b + MB : nullptr;
  if (!cur_b) return stp_fail(ctx, STP_ENOSPACE, "out of host memory%s");
  for (size_t i = 0; i < n_ops; i++) {
    const stp_op &o = ops[i];
    if (o.kind == STP_OP_F) f_mb = o.microbatch;
    if (o.kind == STP_OP_B || o.kind == STP_OP_BW) cur_b[o.microbatch] = 1;
    if (o.kind == STP_OP_W || o.kind == STP_OP_BW) cur_w[o.microbatch] = 1;
  }
  // Joins with the steps before.  Data of a (layer, microbatch) is written by that microbatch's F units (forward
  // stream), read and extended by its B units (backward stream), read by its W units (weight-gradient stream);
  // gradient accumulators and workspace lanes belong to one stream each.  So, of the last step, a stream waits
  // only for   F: the B / W streams if they worked on the microbatch this step's F overwrites;
  //            B: the F stream if it produced one of this step's backward microbatches, the W stream if it read one;
  //            W: the B stream if it produced what this step's W units read (and the F stream likewise).
  // All streams wait for the whole of the step before last, which bounds the skew to one block.  If the caller
  // changed streams, or the stage's extent changed, every stream waits for everything.
  const int last = ctx->ev_gen ^ 1, older = ctx->ev_gen;
  bool same_streams = ctx->ev_valid[last] && ctx->last_mbs == MB && ctx->last_b;
  for (int i = 0; i < 3 && same_streams; i++) same_streams = ctx->ev_stream[last][i] == streams[i];
  auto wait_for = [&](hipStream_t s, int gen, int j) -> int {
    if (!ctx->ev_valid[gen] || ctx->ev_stream[gen][j] == s) return STP_OK;
    STP_HIP(ctx, hipStreamWaitEvent(s, ctx->ev_step[gen][ctx->ev_alias[gen][j]], 0));
    return STP_OK;
  };
  rc = STP_OK;
  if (ctx->ev_next && !same_streams) {
    for (int i = 0; i < 3 && rc == STP_OK; i++) {
      if (i > 0 && (streams[i] == streams[i - 1] || streams[i] == streams[0])) continue;   // already joined
      for (int g = 0; g < 2; g++)
        for (int j = 0; j < 3 && rc == STP_OK; j++) rc = wait_for(streams[i], g, j);
    }
  } else if (ctx->ev_next && !serial) {
    for (int i = 0; i < 3 && rc == STP_OK; i++)
      for (int j = 0; j < 3 && rc == STP_OK; j++) rc = wait_for(streams[i], older, j);
    bool b_after_f = false, b_after_w = false, w_after_b = false, w_after_f = false;
    for (int m = 0; m < MB; m++) {
      if (cur_b[m] && m == ctx->last_f_mb) b_after_f = true;
      if (cur_b[m] && ctx->last_w[m]) b_after_w = true;
      if (cur_w[m] && ctx->last_b[m]) w_after_b = true;
      if (cur_w[m] && m == ctx->last_f_mb) w_after_f = true;
    }
    if (rc == STP_OK && f_mb >= 0 && ctx->last_b[f_mb]) rc = wait_for(sF, last, 1);
    if (rc == STP_OK && f_mb >= 0 && ctx->last_w[f_mb]) rc = wait_for(sF, last, 2);
    if (rc == STP_OK && b_after_f) rc = wait_for(sB, last, 0);
    if (rc == STP_OK && b_after_w) rc = wait_for(sB, last, 2);
    if (rc == STP_OK && w_after_b) rc = wait_for(sW, last, 1);
    if (rc == STP_OK && w_after_f) rc = wait_for(sW, last, 0);
  }
  if (rc != STP_OK) { free(cur_b); return rc; }
  int *ev_of = (int *)malloc(sizeof(int) * bsz);
  uint8_t *b_now = (uint8_t *)calloc(bsz, 1);      // B units issued by this step; committed to the context when the step is whole
  if (!ev_of || !b_now) { free(ev_of); free(b_now); free(cur_b); return stp_fail(ctx, STP_ENOSPACE, "out of host memory%s"); }
  for (size_t i = 0; i < bsz; i++) ev_of[i] = -1;
  int ev_used = 0;
  rc = STP_OK;
  // The GEMMs choose their tile differently when other streams share the GPU: that is so when this step puts
  // work on at least two different streams (a block of forward passes only, or of stored W units only, runs alone).
  {
    bool any_b = false, any_w = false;
    for (int m = 0; m < MB; m++) { any_b = any_b || cur_b[m]; any_w = any_w || cur_w[m]; }
    hipStream_t used[3]; int nu = 0;
    auto use = [&](hipStream_t s) { for (int i = 0; i < nu; i++) if (used[i] == s) return; used[nu++] = s; };
    if (f_mb >= 0) use(sF);
    if (any_b) use(sB);
    if (any_w) use(sW);
    ctx->concurrent = nu >= 2 ? 1 : 0;
  }

  for (size_t i = 0; i < n_ops && rc == STP_OK; i++) {
    const stp_op &o = ops[i];
    const stp_layer_desc *d = &st->desc[o.layer];
    const stp_weights *w = &st->w[o.layer];
    stp_wgrads *g = &st->g[o.layer];
    // Each accumulator goes to exactly one unit.  The bias gradients of the row-parallel linears (b_o, b_fc2: 1/t
    // of the column sum of the unit's upstream gradient) ride in the norm backward of the Pre-* B unit below
    // them, which reads that gradient anyway; the W units get a table without them.
    stp_wgrads g_b, g_w = *g;
    memset(&g_b, 0, sizeof(g_b));
    g_b.norm1_g = g->norm1_g; g_b.norm1_b = g->norm1_b; g_b.norm2_g = g->norm2_g; g_b.norm2_b = g->norm2_b;
    g_b.b_o = g->b_o; g_b.b_fc2 = g->b_fc2;
    g_w.b_o = nullptr; g_w.b_fc2 = nullptr;
    const stp_stash *stash = &st->stash[(size_t)o.layer * MB + o.microbatch];
    size_t off[STP_ST_NFIELDS], nbytes;
    for (int f = 0; f < STP_ST_NFIELDS; f++) stp_stash_field(d, f, &off[f], &nbytes);
    char *sb = (char *)stash->base;
    void *x = st->act[(size_t)o.layer * MB + o.microbatch];
    // a layer that ends a chain in the middle of the stage has its own output / upstream-gradient slots
    const bool tail = o.layer + 1 < L && st->chain_break && st->chain_break[o.layer + 1];
    void *x_out = tail ? st->tail_act[(size_t)o.layer * MB + o.microbatch] : st->act[(size_t)(o.layer + 1) * MB + o.microbatch];
    void *dx = st->grad[(size_t)o.layer * MB + o.microbatch];
    void *dx_out = tail ? st->tail_grad[(size_t)o.layer * MB + o.microbatch] : st->grad[(size_t)(o.layer + 1) * MB + o.microbatch];
    void *x_attn = sb + off[STP_ST_X_ATTN], *dx_attn = sb + off[STP_ST_DX_ATTN];
    void *dz = sb + off[STP_ST_DZ], *dx_ln = sb + off[STP_ST_DX_LN];
    const size_t act_bytes = (size_t)d->seq * d->mbsz * d->hidden * stp_elem_size(d->dtype);
    const size_t slot = ((size_t)o.layer * MB + o.microbatch) * 2 + (o.unit == STP_MLP ? 1 : 0);
    const bool has_w = o.unit == STP_ATTN || o.unit == STP_MLP;

    if (o.kind == STP_OP_F) {
      switch (o.unit) {
        case STP_PRE_ATTN: rc = stp_forward_unit(ctx, d, o.unit, w, x, nullptr, nullptr, stash, 0, sF); break;
        case STP_ATTN:
          rc = stp_forward_unit(ctx, d, o.unit, w, nullptr, x, x_attn, stash, 0, sF);
          if (rc == STP_OK && cb) cb(user, STP_AR_F_ATTN, x_attn, act_bytes, o.layer, o.microbatch, sF);
          break;
        case STP_PRE_MLP: rc = stp_forward_unit(ctx, d, o.unit, w, x_attn, nullptr, nullptr, stash, 0, sF); break;
        case STP_MLP:
          rc = stp_forward_unit(ctx, d, o.unit, w, nullptr, x_attn, x_out, stash, 0, sF);
          if (rc == STP_OK && cb) cb(user, STP_AR_F_MLP, x_out, act_bytes, o.layer, o.microbatch, sF);
          break;
      }
      continue;
    }
    if (o.kind == STP_OP_B || o.kind == STP_OP_BW) {
      switch (o.unit) {
        case STP_MLP:
          rc = stp_backward_input_unit(ctx, d, o.unit, w, stash, nullptr, dx_out, nullptr, dz, nullptr, 1, sB);
          if (rc == STP_OK && cb) cb(user, STP_AR_B_MLP, dz, act_bytes, o.layer, o.microbatch, sB);
          break;
        case STP_PRE_MLP: rc = stp_backward_input_unit(ctx, d, o.unit, w, stash, x_attn, dz, dx_out, dx_attn, &g_b, 1, sB); break;
        case STP_ATTN:
          rc = stp_backward_input_unit(ctx, d, o.unit, w, stash, nullptr, dx_attn, nullptr, dx_ln, nullptr, 1, sB);
          if (rc == STP_OK && cb) cb(user, STP_AR_B_ATTN, dx_ln, act_bytes, o.layer, o.microbatch, sB);
          break;
        case STP_PRE_ATTN: rc = stp_backward_input_unit(ctx, d, o.unit, w, stash, x, dx_ln, dx_attn, dx, &g_b, 1, sB); break;
      }
      if (rc != STP_OK) break;
      if (has_w) {
        b_now[slot] = 1;
        if (!serial && sW != sB) {
          hipError_t e = hipEventRecord(ctx->ev_pool[ev_used], sB);
          if (e != hipSuccess) { rc = stp_fail(ctx, STP_EHIP, "hipEventRecord failed: %s", hipGetErrorString(e)); break; }
          ev_of[slot] = ev_used++;
        }
      }
    }
    if ((o.kind == STP_OP_W || o.kind == STP_OP_BW) && has_w) {
      if (!serial && sW != sB && ev_of[slot] >= 0) {
        hipError_t e = hipStreamWaitEvent(sW, ctx->ev_pool[ev_of[slot]], 0);
        if (e != hipSuccess) { rc = stp_fail(ctx, STP_EHIP, "hipStreamWaitEvent failed: %s", hipGetErrorString(e)); break; }
      }
      const void *dy = o.unit == STP_MLP ? dx_out : dx_attn;
      rc = stp_backward_weight_unit(ctx, d, o.unit, stash, dy, &g_w, 2, sW);
    }
  }
  free(ev_of);
  ctx->concurrent = 0;
  // The end-of-step events are recorded on the error path too: whatever part of the step was enqueued, later
  // steps still order themselves behind it.  The B units count as done only when the whole step was issued.
  {
    const int gen = ctx->ev_gen;
    for (int i = 0; i < 3; i++) {      // one event per distinct stream (a serialised step records one)
      ctx->ev_stream[gen][i] = streams[i];
      ctx->ev_alias[gen][i] = i;
      for (int j = 0; j < i; j++)
        if (streams[j] == streams[i]) { ctx->ev_alias[gen][i] = ctx->ev_alias[gen][j]; break; }
      if (ctx->ev_alias[gen][i] != i) continue;
      const hipError_t e = hipEventRecord(ctx->ev_step[gen][i], streams[i]);
      if (e != hipSuccess && rc == STP_OK) rc = stp_fail(ctx, STP_EHIP, "hipEventRecord failed: %s", hipGetErrorString(e));
    }
    ctx->ev_valid[gen] = 1;
    ctx->ev_gen = gen ^ 1;
    if (ctx->last_mbs != MB || !ctx->last_b) {
      free(ctx->last_b);
      ctx->last_b = (uint8_t *)calloc(2 * (size_t)MB, 1);
      ctx->last_w = ctx->last_b ? ctx->last_b + MB : nullptr;
      ctx->last_mbs = ctx->last_b ? MB : 0;
    }
    if (ctx->last_b) memcpy(ctx->last_b, cur_b, 2 * (size_t)MB);
    ctx->last_f_mb = f_mb;
  }
  free(cur_b);
  ctx->ev_next = 1;
  if (rc == STP_OK)
    for (size_t i = 0; i < bsz; i++) ctx->b_done[i] |= b_now[i];
  free(b_now);
  return rc;
}

// Activation offload and reload (Section 4.2, last paragraph; Section 4.3): a fraction alpha of the stashed
// activations that live long (those only a deferred W unit still reads; those a chunk's forward pass leaves
// for its backward pass) is copied to page-locked host memory on a copy stream while the compute streams
// run, and copied back before the unit that needs it.  Host code only: the copies are plain asynchronous
// HIP memory copies, ordered against the producer and consumer streams by events.
#include "common.h"

namespace {

constexpr size_t GRANULE = 256;   // copies move whole 256-byte pieces (every stash field starts on one)

int set_fields(const stp_layer_desc *d, int set, int (&fields)[STP_ST_NFIELDS]) {
  const bool sw = d->act == STP_ACT_SWIGLU;
  int n = 0;
  switch (set) {
    case STP_OFFLOAD_W_ATTN:
      fields[n++] = STP_ST_X_LN; fields[n++] = STP_ST_CTX; fields[n++] = STP_ST_DQKV;
      break;
    case STP_OFFLOAD_W_MLP:
      fields[n++] = STP_ST_Z_LN; fields[n++] = STP_ST_G; fields[n++] = STP_ST_DH;
      if (sw) fields[n++] = STP_ST_DHU;
      break;
    case STP_OFFLOAD_FWD:
      fields[n++] = STP_ST_X_LN; fields[n++] = STP_ST_STATS1; fields[n++] = STP_ST_QKV; fields[n++] = STP_ST_CTX;
      fields[n++] = STP_ST_LSE; fields[n++] = STP_ST_Z_LN; fields[n++] = STP_ST_STATS2; fields[n++] = STP_ST_H;
      if (sw) fields[n++] = STP_ST_HU;
      fields[n++] = STP_ST_G; fields[n++] = STP_ST_X_ATTN;
      break;
    default: return -1;
  }
  return n;
}

struct Segment { size_t dev_off, host_off, bytes; };

// the leading share of every field of the set; returns the number of segments, or -1
int plan(const stp_layer_desc *d, int set, float alpha, Segment (&seg)[STP_ST_NFIELDS], size_t *total) {
  if (!d || !(alpha >= 0.f && alpha <= 1.f)) return -1;
  if (stp_check_desc(d) != STP_OK) return -1;
  int fields[STP_ST_NFIELDS];
  const int nf = set_fields(d, set, fields);
  if (nf < 0) return -1;
  size_t host_off = 0;
  int n = 0;
  for (int i = 0; i < nf; i++) {
    size_t off, bytes;
    if (stp_stash_field(d, fields[i], &off, &bytes) != STP_OK) return -1;
    // alpha * bytes in double: exact for alpha = 1 and monotone in alpha
    size_t want = (size_t)((double)alpha * (double)bytes);
    if ((double)want < (double)alpha * (double)bytes) want++;
    size_t take = stp_align_up(want, GRANULE);
    if (take > bytes) take = bytes;
    if (take == 0) continue;
    seg[n++] = {off, host_off, take};
    host_off += take;
  }
  *total = host_off;
  return n;
}

int next_event(stp_ctx *ctx, hipEvent_t *ev) {
  const int cap = (int)(sizeof(ctx->ev_copy) / sizeof(ctx->ev_copy[0]));
  const int idx = ctx->ev_copy_next;          // idx <= ev_copy_made: the ring fills in order
  if (idx == ctx->ev_copy_made) {
    STP_HIP(ctx, hipEventCreateWithFlags(&ctx->ev_copy[idx], hipEventDisableTiming));
    ctx->ev_copy_made++;
  }
  *ev = ctx->ev_copy[idx];
  ctx->ev_copy_next = (idx + 1) % cap;
  return STP_OK;
}

}  // namespace

extern "C" int stp_offload_bytes(const stp_layer_desc *d, int set, float alpha, size_t *bytes) {
  if (!bytes) return STP_EINVAL;
  Segment seg[STP_ST_NFIELDS];
  size_t total = 0;
  if (plan(d, set, alpha, seg, &total) < 0) return STP_EINVAL;
  *bytes = total;
  return STP_OK;
}

extern "C" int stp_stash_offload(stp_ctx *ctx, const stp_layer_desc *d, int set, float alpha, const stp_stash *stash,
                                 void *host, size_t host_bytes, void *s_producer, void *s_copy) {
  if (!ctx) return STP_EINVAL;
  if (!stash || !stash->base || !host) return stp_fail(ctx, STP_EINVAL, "stp_stash_offload: null pointer%s");
  Segment seg[STP_ST_NFIELDS];
  size_t total = 0, need = 0;
  const int n = plan(d, set, alpha, seg, &total);
  if (n < 0) return stp_fail(ctx, STP_EINVAL, "stp_stash_offload: bad layer description, set or alpha%s");
  if (host_bytes < total)
    return stp_fail(ctx, STP_EINVAL, "stp_stash_offload: host buffer too small%s (need %ld bytes)", "", (long)total);
  if (stp_stash_bytes(d, &need) != STP_OK || stash->bytes < need)
    return stp_fail(ctx, STP_EINVAL, "stp_stash_offload: stash too small%s (need %ld bytes)", "", (long)need);
  hipStream_t sp = (hipStream_t)s_producer, sc = (hipStream_t)s_copy;
  if (sp != sc) {
    hipEvent_t ev;
    int rc = next_event(ctx, &ev);
    if (rc != STP_OK) return rc;
    STP_HIP(ctx, hipEventRecord(ev, sp));
    STP_HIP(ctx, hipStreamWaitEvent(sc, ev, 0));
  }
  for (int i = 0; i < n; i++)
    STP_HIP(ctx, hipMemcpyAsync((char *)host + seg[i].host_off, (const char *)stash->base + seg[i].dev_off, seg[i].bytes,
                                hipMemcpyDeviceToHost, sc));
  return STP_OK;
}

extern "C" int stp_stash_reload(stp_ctx *ctx, const stp_layer_desc *d, int set, float alpha, const stp_stash *stash,
                                const void *host, size_t host_bytes, void *s_copy, void *s_consumer) {
  if (!ctx) return STP_EINVAL;
  if (!stash || !stash->base || !host) return stp_fail(ctx, STP_EINVAL, "stp_stash_reload: null pointer%s");
  Segment seg[STP_ST_NFIELDS];
  size_t total = 0, need = 0;
  const int n = plan(d, set, alpha, seg, &total);
  if (n < 0) return stp_fail(ctx, STP_EINVAL, "stp_stash_reload: bad layer description, set or alpha%s");
  if (host_bytes < total)
    return stp_fail(ctx, STP_EINVAL, "stp_stash_reload: host buffer too small%s (need %ld bytes)", "", (long)total);
  if (stp_stash_bytes(d, &need) != STP_OK || stash->bytes < need)
    return stp_fail(ctx, STP_EINVAL, "stp_stash_reload: stash too small%s (need %ld bytes)", "", (long)need);
  hipStream_t sc = (hipStream_t)s_copy, su = (hipStream_t)s_consumer;
  for (int i = 0; i < n; i++)
    STP_HIP(ctx, hipMemcpyAsync((char *)stash->base + seg[i].dev_off, (const char *)host + seg[i].host_off, seg[i].bytes,
                                hipMemcpyHostToDevice, sc));
  if (su != sc) {
    hipEvent_t ev;
    int rc = next_event(ctx, &ev);
    if (rc != STP_OK) return rc;
    STP_HIP(ctx, hipEventRecord(ev, sc));
    STP_HIP(ctx, hipStreamWaitEvent(su, ev, 0));
  }
  return STP_OK;
}

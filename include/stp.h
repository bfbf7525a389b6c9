/*
 * stp.h - C ABI of the braided F/B/W computation units of one tensor-parallel
 * shard of a transformer layer, for one AMD MI355X (gfx950).
 *
 * The decomposition follows the paper "Synergistic Tensor and Pipeline
 * Parallelism": a layer is cut into the Pre-Attn, Attn, Pre-MLP and MLP units
 * (Section 3); the residual add is folded into the Attn / MLP unit before the
 * TP reduction, each of the t ranks adding X/t (Eq. 1) and the backward taking
 * an un-reduced "+1" path (Eq. 2); the backward of Attn and MLP is split into
 * an activation-gradient part B and a weight-gradient part W (Section 3); a
 * braided block interleaves the F units of microbatch i with the B/W units of
 * a microbatch j < i (Section 3, Section 4.1 pattern (2), Appendix A).
 *
 * Conventions for every entry point
 *   - returns an stp_status; never throws, aborts or prints;
 *   - "device" pointers are HIP device memory owned by the CALLER, 16-byte
 *     aligned, row-major contiguous; activations are [tokens, features] with
 *     tokens = seq * mbsz; linear weights are [in_features, out_features];
 *     w_qkv columns are [Q heads | K heads | V heads], head-major;
 *   - element type of activations and weights is desc->dtype (fp32 or bf16);
 *     weight-gradient accumulators are ALWAYS fp32, are accumulated into
 *     ("+="), and are zeroed by the caller;
 *   - streams are raw hipStream_t handles passed as void*; calls only enqueue
 *     work and return; a device fault surfaces as STP_EHIP on a later call or
 *     at the caller's synchronisation;
 *   - the library owns only the context (events, small tables) and uses the
 *     caller-supplied workspace; it never allocates device memory;
 *   - a context is for one host thread at a time (it carries the last error
 *     text, the braid's bookkeeping and the event ring of the offload calls),
 *     and a process uses the library on one device: kernel attributes that the
 *     launchers set once per process are set on the device current then;
 *   - the four points per layer where a TP All-Reduce would fall (after Attn
 *     and MLP in forward, after MLP-B and Attn-B in backward; Section 3) are
 *     boundaries: unit outputs there are this rank's PARTIAL and the caller
 *     (or the boundary callback of stp_braid_step) owns the reduction.
 */
#ifndef STP_H_
#define STP_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct stp_ctx stp_ctx; /* opaque, library-owned, one per device */

typedef enum {
  STP_OK = 0,
  STP_EINVAL = 1,       /* null pointer, bad enum value */
  STP_ESHAPE = 2,       /* a dimension the kernels cannot take (see stp_check_desc) */
  STP_EALIGN = 3,       /* pointer not 16-byte aligned */
  STP_ENOSPACE = 4,     /* stash or workspace smaller than stp_*_bytes says */
  STP_ESEQ = 5,         /* op list violates the braid's ordering rules */
  STP_EUNSUPPORTED = 6,
  STP_EHIP = 7          /* a HIP runtime call failed; see stp_last_error */
} stp_status;

/* The four fine-grained units of a layer (Section 3). */
typedef enum { STP_PRE_ATTN = 0, STP_ATTN = 1, STP_PRE_MLP = 2, STP_MLP = 3 } stp_unit;

/* F forward, B activation gradient, W weight gradient, BW = B immediately
 * followed by its W ("full backward", Fig. 3a; W separation off, Section 4.2). */
typedef enum { STP_OP_F = 0, STP_OP_B = 1, STP_OP_W = 2, STP_OP_BW = 3 } stp_opkind;

typedef enum { STP_F32 = 0, STP_BF16 = 1 } stp_dtype;
typedef enum { STP_NORM_LN = 0, STP_NORM_RMS = 1 } stp_norm;
typedef enum { STP_ACT_GELU = 0, STP_ACT_SWIGLU = 1 } stp_act;

/* The TP boundaries (f / g operators of Fig. 2). */
typedef enum { STP_AR_F_ATTN = 0, STP_AR_F_MLP = 1, STP_AR_B_MLP = 2, STP_AR_B_ATTN = 3 } stp_boundary;

/* One rank's share of a layer and the microbatch shape. */
typedef struct {
  int32_t hidden;       /* h, multiple of 8 */
  int32_t heads_local;  /* n, heads on this rank */
  int32_t head_dim;     /* d, 64 or 128 for bf16; any multiple of 8 up to 128 for fp32 */
  int32_t ffn_local;    /* f, FFN columns on this rank, multiple of 8 */
  int32_t seq;          /* tokens per sequence */
  int32_t mbsz;         /* sequences per microbatch (tokens = seq * mbsz) */
  int32_t tp;           /* t of Eq. 1: residual and row-parallel biases enter as 1/t */
  int32_t dtype;        /* stp_dtype of activations and weights */
  int32_t norm;         /* stp_norm */
  int32_t act;          /* stp_act */
  int32_t causal;       /* 1: key j > query i is masked */
  int32_t rope;         /* 1: rotate-half rotary embedding on Q and K, positions 0..seq-1 */
  int32_t has_bias;     /* 1: linear layers carry biases */
  float eps;            /* norm epsilon */
  float rope_base;      /* e.g. 10000 */
  int32_t kv_heads_local; /* key / value heads on this rank (grouped-query attention: the model table of Section 5.1
                           * lists 40 / 8 and 56 / 8 query / key-value heads); 0 = heads_local; must divide heads_local.
                           * QKV activations are [tokens][(heads_local + 2 kv_heads_local) head_dim]: Q heads, K heads, V heads */
} stp_layer_desc;

/* Device pointers to one rank's weights; entries a configuration does not use
 * may be NULL (norm*_b for RMSNorm, b_* when has_bias = 0, w_up for GELU). */
typedef struct {
  const void *norm1_g, *norm1_b; /* [h] */
  const void *w_qkv, *b_qkv;     /* [h, c], [c]   c = (n + 2 n_kv) d: Q heads | K heads | V heads; a = n*d */
  const void *w_o, *b_o;         /* [a, h],  [h]   (row-parallel: bias enters as b_o/t) */
  const void *norm2_g, *norm2_b; /* [h] */
  const void *w_fc1, *b_fc1;     /* [h, f],  [f]   (SwiGLU: the gate projection) */
  const void *w_up;              /* [h, f]         (SwiGLU only) */
  const void *w_fc2, *b_fc2;     /* [f, h],  [h]   (row-parallel: b_fc2/t) */
} stp_weights;

/* fp32 gradient accumulators, same shapes as stp_weights; NULL entries are skipped. */
typedef struct {
  float *norm1_g, *norm1_b, *w_qkv, *b_qkv, *w_o, *b_o;
  float *norm2_g, *norm2_b, *w_fc1, *b_fc1, *w_up, *w_fc2, *b_fc2;
} stp_wgrads;

/* Per (layer, microbatch) device buffer holding what F leaves for B and W and
 * what B leaves for W.  Size from stp_stash_bytes; field offsets from
 * stp_stash_field.  Caller-owned; contents are library-defined. */
typedef struct { void *base; size_t bytes; } stp_stash;

typedef enum {
  STP_ST_X_LN = 0,   /* [T, h]   Pre-Attn output                          */
  STP_ST_STATS1,     /* [T, 2]   fp32 (mean, rstd) of Pre-Attn            */
  STP_ST_QKV,        /* [T, c]   Q|K|V after bias and RoPE                */
  STP_ST_CTX,        /* [T, a]   attention output before the out-proj     */
  STP_ST_LSE,        /* [mbsz, n, seq] fp32 log-sum-exp of the score rows */
  STP_ST_Z_LN,       /* [T, h]   Pre-MLP output                           */
  STP_ST_STATS2,     /* [T, 2]   fp32                                     */
  STP_ST_H,          /* [T, f]   FC1 pre-activation (SwiGLU: gate)        */
  STP_ST_HU,         /* [T, f]   SwiGLU up projection                     */
  STP_ST_G,          /* [T, f]   activation output, input of FC2          */
  STP_ST_DH,         /* [T, f]   written by MLP-B, read by MLP-W          */
  STP_ST_DHU,        /* [T, f]   SwiGLU only                              */
  STP_ST_DG,         /* [T, f]   scratch of MLP-B (SwiGLU only)           */
  STP_ST_DQKV,       /* [T, c]   written by Attn-B, read by Attn-W        */
  STP_ST_DCTX,       /* [T, a]   scratch of Attn-B                        */
  STP_ST_DELTA,      /* [mbsz, n, seq] fp32 rowsum(dctx * ctx)            */
  STP_ST_X_ATTN,     /* [T, h]   used by stp_braid_step: Attn output      */
  STP_ST_DX_ATTN,    /* [T, h]   used by stp_braid_step                   */
  STP_ST_DZ,         /* [T, h]   used by stp_braid_step: MLP-B output     */
  STP_ST_DX_LN,      /* [T, h]   used by stp_braid_step: Attn-B output    */
  STP_ST_NFIELDS
} stp_stash_field_id;

/* One entry of a braided sequence. */
typedef struct { int32_t kind /* stp_opkind */, unit /* stp_unit */, layer, microbatch; } stp_op;

/* One PP stage's model chunk and its in-flight microbatches (Section 4.2). */
typedef struct {
  int32_t n_layers, n_microbatches;
  const stp_layer_desc *desc; /* [n_layers]; layers may differ (ViT + LM stage) */
  const stp_weights *w;       /* [n_layers] */
  stp_wgrads *g;              /* [n_layers] */
  stp_stash *stash;           /* [n_layers * n_microbatches], index layer*n_microbatches + mb */
  void **act;                 /* [(n_layers+1) * n_microbatches]: act[l*M+mb] = input of layer l,
                                 act[n_layers*M+mb] = stage output.  A layer's output must have the
                                 next layer's input shape unless chain_break[l+1] is set. */
  void **grad;                /* same indexing: gradient w.r.t. act[...] */
  const int32_t *chain_break; /* NULL, or [n_layers+1]: chain_break[l] = 1 means layer l starts a new
                                 chain: act[l*M+mb] is that chain's own input (grad[l*M+mb] receives its
                                 input gradient), and layer l-1, which ends the previous chain, writes its
                                 output to tail_act[(l-1)*M+mb] and reads its upstream gradient from
                                 tail_grad[(l-1)*M+mb] instead */
  void **tail_act;            /* [n_layers * n_microbatches]; only entries of chain-ending interior layers
                                 are used; may be NULL when chain_break has no interior 1 */
  void **tail_grad;           /* same indexing */
} stp_stage;

/* Called on the issuing stream's behalf at every TP boundary inside
 * stp_braid_step: `buf` holds this rank's partial of `bytes` bytes, produced by
 * work already enqueued on `hip_stream`; whatever the callback enqueues on that
 * stream (e.g. an all-reduce) is ordered before the consumer unit. */
typedef void (*stp_boundary_fn)(void *user, int which /* stp_boundary */, void *buf, size_t bytes,
                                int32_t layer, int32_t microbatch, void *hip_stream);

/* ---- context ------------------------------------------------------------ */
int stp_create(stp_ctx **out, int device);
int stp_destroy(stp_ctx *ctx);
const char *stp_last_error(const stp_ctx *ctx);
const char *stp_status_str(int status);

/* Checks that the kernels can take this shape (STP_ESHAPE / STP_EINVAL otherwise). */
int stp_check_desc(const stp_layer_desc *desc);
int stp_stash_bytes(const stp_layer_desc *desc, size_t *bytes);
int stp_stash_field(const stp_layer_desc *desc, int field, size_t *offset, size_t *bytes);
/* Workspace (norm-gradient and column-sum partials, attention chunk partials) for three concurrent
 * streams; the maximum over the layers of a stage must be supplied. */
int stp_workspace_bytes(const stp_layer_desc *desc, size_t *bytes);
int stp_set_workspace(stp_ctx *ctx, void *device_ptr, size_t bytes);

/* ---- the units (Section 3; Eq. 1-2) --------------------------------------
 * lane selects the third of the workspace the call may use (0, 1 or 2); two
 * calls that may run concurrently must use different lanes.
 *
 * stp_forward_unit
 *   PRE_ATTN: x_in = X [T,h]                   -> stash X_LN, STATS1      (y_out unused)
 *   ATTN    : x_resid = X                      -> y_out = this rank's partial of X_attn;
 *             stash QKV, CTX, LSE.  y = ctx*Wo + b_o/t + X/t   (Eq. 1)
 *   PRE_MLP : x_in = X_attn (reduced)          -> stash Z_LN, STATS2
 *   MLP     : x_resid = X_attn                 -> y_out = partial of the layer output;
 *             stash H, G (and HU)
 */
int stp_forward_unit(stp_ctx *ctx, const stp_layer_desc *desc, int unit, const stp_weights *w,
                     const void *x_in, const void *x_resid, void *y_out, const stp_stash *stash,
                     int lane, void *hip_stream);

/* stp_backward_input_unit (activation gradients, "B")
 *   MLP     : dy = dX_out                      -> dx = partial of dZ_ln; stash DH (DHU)
 *   PRE_MLP : x_in = X_attn, dy = dZ_ln (reduced), d_resid = dX_out
 *                                              -> dx = dX_attn = norm_bwd(dy) + d_resid (Eq. 2)
 *                                                 norm gain/bias grads += into wg (may be NULL)
 *   ATTN    : dy = dX_attn                     -> dx = partial of dX_ln; stash DQKV
 *   PRE_ATTN: x_in = X, dy = dX_ln (reduced), d_resid = dX_attn -> dx = dX
 * Of `wg` the Pre-* units use the four norm entries and ONE bias entry: d_resid is the upstream gradient of
 * the MLP (PRE_MLP) / Attn (PRE_ATTN) unit above, so (1/t) of its column sum is that unit's row-parallel bias
 * gradient; the unit reads d_resid anyway and adds it into wg->b_fc2 (PRE_MLP) / wg->b_o (PRE_ATTN) when that
 * entry is non-NULL and the layer has biases.  The W unit adds the same quantity when ITS table holds the
 * entry: hand each accumulator to exactly one of the two (stp_braid_step gives b_fc2 / b_o to the Pre-* units).
 */
int stp_backward_input_unit(stp_ctx *ctx, const stp_layer_desc *desc, int unit, const stp_weights *w,
                            const stp_stash *stash, const void *x_in, const void *dy,
                            const void *d_resid, void *dx, stp_wgrads *wg, int lane, void *hip_stream);

/* stp_backward_weight_unit (weight gradients, "W"; needs the unit's B to have run)
 *   MLP : dy = dX_out   -> w_fc2 += G^T dy, w_fc1 += Z_ln^T dH, (w_up), b_fc1 += sum dH, b_fc2 += sum dy / t
 *   ATTN: dy = dX_attn  -> w_o += ctx^T dy, w_qkv += X_ln^T dQKV, b_qkv += sum dQKV, b_o += sum dy / t
 */
int stp_backward_weight_unit(stp_ctx *ctx, const stp_layer_desc *desc, int unit, const stp_stash *stash,
                             const void *dy, stp_wgrads *wg, int lane, void *hip_stream);

/* ---- the braided block (Section 3, Fig. 3; Section 4.1 pattern (2); Appendix A)
 * Issues `ops` in the given order: F ops on s_fwd, B ops on s_bwd, W ops (and
 * the W half of BW ops) on s_wgrad, with events only on true data dependences:
 * a W waits for its B; of the previous step, a stream waits only for the streams
 * whose work it reads or overwrites (the forward stream for B / W work on the
 * microbatch whose stash it refills, the backward stream for the forward pass of
 * its microbatches and for W work on them, the weight-gradient stream for their
 * B units), and every stream waits for the whole of the step before that: at
 * most two blocks are in flight, and a block's tail overlaps the next one's head.
 * (Gradient accumulators and workspace lanes are touched by one stream each;
 * units called directly on other streams are the caller's to order.)  The list is
 * validated first (STP_ESEQ): all F ops belong to one microbatch i, all B / W /
 * BW ops to microbatches j < i (Appendix A) unless the list has no F op; units
 * of one direction appear in dependence order; a W op needs its B in this list
 * or in an earlier step.  Passing the same stream three times serialises the
 * step (used to check braided == sequential bit for bit).  If the streams differ
 * from the previous step's, every stream waits for the whole of the steps before:
 * the streams may change from one step to the next without a synchronisation by
 * the caller.
 * STP_ESHAPE: two consecutive layers with no chain break between them differ in
 * tokens (seq * mbsz), hidden or dtype (the first writes into the second's input
 * slot).  STP_EUNSUPPORTED: one of the streams is being captured into a HIP graph.
 * Every host-side condition of the list is checked before the first launch; B
 * units count as run (for later W ops) only when the whole step was issued. */
int stp_braid_step(stp_ctx *ctx, const stp_stage *stage, const stp_op *ops, size_t n_ops,
                   void *s_fwd, void *s_bwd, void *s_wgrad, stp_boundary_fn cb, void *user);
/* Validation alone (host only, no GPU needed); *bad_index gets the offending op. */
int stp_validate_ops(const stp_stage *stage, const stp_op *ops, size_t n_ops, size_t *bad_index);
/* Forget which B units earlier steps have run (start of a new iteration). */
int stp_braid_reset(stp_ctx *ctx);
/* The next stp_braid_step does not wait for the step before it: for a caller that has ordered the three
 * streams itself since then (a device synchronisation, say).
 * Stream capture: recording three-stream steps into a HIP graph is NOT supported (the one attempt crashed the
 * host process inside the runtime when the capture ended, and the cause is not known); stp_braid_step returns
 * STP_EUNSUPPORTED when any of its streams is capturing. */
int stp_braid_detach(stp_ctx *ctx);

/* ---- activation offload and reload (Section 4.2, last paragraph; Section 4.3) --------------------
 * The schedule keeps some stashed activations for a long time: those of a microbatch whose weight
 * gradients are separated from its backward pass and deferred, and those of model chunk 0 between its
 * forward and its backward pass.  A fraction alpha of them is copied to host memory on a copy stream, in
 * parallel with the compute streams, and copied back before the unit that reads them.
 *
 * `set` names the group of stash fields:
 *   STP_OFFLOAD_W_ATTN  what only Attn-W still reads once Attn-B has run:  X_LN, CTX, DQKV
 *   STP_OFFLOAD_W_MLP   what only MLP-W still reads once MLP-B has run:    Z_LN, G, DH (DHU)
 *   STP_OFFLOAD_FWD     what the forward units leave for the backward side:
 *                       X_LN, STATS1, QKV, CTX, LSE, Z_LN, STATS2, H, (HU), G, X_ATTN
 * Of every field of the set the leading ceil(alpha * bytes / 256) * 256 bytes (at most the field) move;
 * their copies lie back to back in `host`, in the order above.  stp_offload_bytes gives their total.
 *
 * stp_stash_offload enqueues: s_copy waits for the work enqueued so far on s_producer, then device -> host
 * copies on s_copy.  Once s_copy has passed them the moved device ranges are dead until reloaded and the
 * caller may reuse them.  stp_stash_reload enqueues the host -> device copies on s_copy and makes
 * s_consumer wait for them.  `host` is host memory of at least stp_offload_bytes bytes, owned by the
 * caller, and must stay untouched between the two calls; it should be page-locked (hipHostMalloc),
 * otherwise the copies do not overlap the compute streams.  alpha outside [0, 1], an unknown set, a NULL
 * pointer or a host buffer that is too small: STP_EINVAL.  A failing HIP call: STP_EHIP. */
typedef enum { STP_OFFLOAD_W_ATTN = 0, STP_OFFLOAD_W_MLP = 1, STP_OFFLOAD_FWD = 2 } stp_offload_set;
int stp_offload_bytes(const stp_layer_desc *desc, int set, float alpha, size_t *bytes);
int stp_stash_offload(stp_ctx *ctx, const stp_layer_desc *desc, int set, float alpha, const stp_stash *stash,
                      void *host, size_t host_bytes, void *s_producer, void *s_copy);
int stp_stash_reload(stp_ctx *ctx, const stp_layer_desc *desc, int set, float alpha, const stp_stash *stash,
                     const void *host, size_t host_bytes, void *s_copy, void *s_consumer);

/* ---- the kernels the units are built from, exposed for per-kernel parity and
 * roofline measurement.  All pointers are device pointers. ------------------ */

/* C[M,N] = op(A) * op(B) with fp32 accumulation; a_trans / b_trans give the storage
 * order of each operand (the weight-gradient GEMMs of the W units contract over the
 * token index, which is the outer index of both of their operands).  Requirements:
 * M, N, K, all leading dimensions multiples of 8; pointers 16-byte aligned. */
typedef struct {
  int32_t dtype;           /* element type of A, B (and of C unless c_f32_accum) */
  int32_t M, N, K;
  const void *A; int32_t lda; int32_t a_trans; /* a_trans=0: A[m*lda+k]; 1: A[k*lda+m] */
  const void *B; int32_t ldb; int32_t b_trans; /* b_trans=0: B[k*ldb+n]; 1: B[n*ldb+k] */
  void *C; int32_t ldc;
  int32_t c_f32_accum;     /* 1: C is fp32 and C += result (weight gradients) */
  const void *bias; float bias_scale;   /* [N] added as bias*bias_scale, or NULL */
  const void *resid; int32_t ldr; float resid_scale; /* [M,N] added as resid*resid_scale, or NULL */
  int32_t epilogue;        /* 0 none; 1: C = v and C2 = gelu(v); 2: C = v * gelu'(aux) */
  void *C2; const void *aux; int32_t ld2;
  int32_t tile_m, tile_n;  /* 0, 0: the library picks the workgroup tile from the shape.  Otherwise each
                            * 128 or 256, or 192 x 256 with a_trans = 0 (bf16 with K a multiple of 32
                            * only): forces that tile, for tuning and tests; anything else is STP_EINVAL */
} stp_gemm_args;
int stp_gemm(stp_ctx *ctx, const stp_gemm_args *args, void *hip_stream);
/* A measured tile preference for the bf16 GEMM of one shape and operand order, used for launches that
 * stp_braid_step issues on concurrent streams (Section 3: the units of a block share the GPU).  Which tile is
 * fastest there depends on the kernels of the other streams; the library's own choice models the GEMM alone.
 * Results do not depend on the tile (every element is summed over K in the same order).  tile_m = tile_n = 0
 * forgets the preference for that shape.  Host only; at most 96 shapes per context (STP_ENOSPACE);
 * STP_EINVAL for a tile stp_gemm_args.tile_m / tile_n would not take. */
int stp_gemm_tile_hint(stp_ctx *ctx, int32_t M, int32_t N, int32_t K, int a_trans, int b_trans,
                       int32_t tile_m, int32_t tile_n);
int stp_gemm_tile_hints_clear(stp_ctx *ctx);

/* Normalisation of the Pre-* units.  stats is fp32 [T,2] (mean, rstd); RMSNorm stores (0, rstd). */
int stp_norm_forward(stp_ctx *ctx, int dtype, int norm, int32_t T, int32_t h, float eps, const void *x,
                     const void *gamma, const void *beta, void *y, float *stats, void *hip_stream);
/* dx = norm_bwd(dy) + d_resid (d_resid may be NULL); dgamma/dbeta (may be NULL) are += .
 * d_resid_sum (may be NULL; needs d_resid): [h] fp32, += d_resid_sum_scale * (sum over the T rows of d_resid). */
int stp_norm_backward(stp_ctx *ctx, int dtype, int norm, int32_t T, int32_t h, const void *x,
                      const void *gamma, const float *stats, const void *dy, const void *d_resid,
                      void *dx, float *dgamma, float *dbeta, float *d_resid_sum, float d_resid_sum_scale,
                      int lane, void *hip_stream);

/* The work plan of one of the chunked bf16 attention kernels for a layer shape (host only, no GPU needed).
 * kind 0: forward, blocks of 128 queries, steps of 128 keys; 1: dK / dV, blocks of 128 keys, steps of 64
 * queries (over every query head of the key head's group); 2: dQ, blocks of 128 queries, steps of 128 keys.
 * A workgroup runs one chunk of at most *chunk_steps consecutive steps of one block; a block has at most
 * *max_chunks chunks (never more than 8), which is what sizes the workspace.  items[0 .. *n_items) are the
 * (block, chunk) pairs in the order the workgroups are dispatched, longest first, as block | chunk << 12;
 * *n_items = 0 means more pairs than the kernel's table holds (1024) and a blocks x chunks grid.  items may
 * be NULL; STP_ENOSPACE if items_cap < *n_items; STP_EUNSUPPORTED for fp32 (those kernels are not chunked). */
int stp_attention_plan(const stp_layer_desc *desc, int kind, int32_t *chunk_steps, int32_t *max_chunks, int32_t *n_items,
                       uint16_t *items, size_t items_cap);

/* Attention core of one rank: qkv is [T, (n + 2 n_kv) d] (n Q heads | n_kv K heads | n_kv V heads; n_kv = n
 * unless desc->kv_heads_local is set), ctx [T, n d], lse fp32 [mbsz,n,seq].  The bf16 kernels cut the key
 * range into chunks whose fp32 partials live in workspace lane `lane` (0..2), and address a sequence's QKV
 * rows with 32-bit byte offsets: seq * (n + 2 n_kv) * d * 2 bytes must stay below 2 GiB (STP_ESHAPE). */
int stp_attention_forward(stp_ctx *ctx, const stp_layer_desc *desc, const void *qkv, void *ctx_out,
                          float *lse, int lane, void *hip_stream);
/* dqkv [T, (n + 2 n_kv) d] from dctx [T, n d]; delta is fp32 scratch [mbsz,n,seq]. */
int stp_attention_backward(stp_ctx *ctx, const stp_layer_desc *desc, const void *qkv, const void *ctx_in,
                           const float *lse, const void *dctx, float *delta, void *dqkv, int lane,
                           void *hip_stream);

/* Elementwise pieces (HBM-bound).  n = number of elements. */
int stp_gelu_forward(stp_ctx *ctx, int dtype, size_t n, const void *x, void *y, void *hip_stream);
int stp_gelu_backward(stp_ctx *ctx, int dtype, size_t n, const void *x, const void *dy, void *dx, void *hip_stream);
int stp_swiglu_forward(stp_ctx *ctx, int dtype, size_t n, const void *gate, const void *up, void *y, void *hip_stream);
int stp_swiglu_backward(stp_ctx *ctx, int dtype, size_t n, const void *gate, const void *up, const void *dy,
                        void *dgate, void *dup, void *hip_stream);
/* Row softmax on its own (the normalisation inside "Attention(.)" of Eq. 1; the attention kernels fuse theirs, this
 * pair is for measuring it against the memory system).  x, y, dy, dx are [rows, n], n a multiple of 8, at most 16384.
 *   forward : y = softmax(scale * x) per row; causal = 1: the rows are stacked [n, n] squares and element j of row r
 *             is masked (y = 0) for j > r mod n
 *   backward: dx = scale * y o (dy - rowsum(dy o y)) */
int stp_softmax_forward(stp_ctx *ctx, int dtype, int32_t rows, int32_t n, float scale, int causal, const void *x, void *y,
                        void *hip_stream);
int stp_softmax_backward(stp_ctx *ctx, int dtype, int32_t rows, int32_t n, float scale, const void *y, const void *dy,
                         void *dx, void *hip_stream);
/* In-place rotary embedding of the Q and K heads of qkv [T, (n + 2 n_kv) d]; inverse = 1 applies the transpose. */
int stp_rope(stp_ctx *ctx, const stp_layer_desc *desc, void *qkv, int inverse, void *hip_stream);
/* out[N] += scale * sum over rows of x[T,N]  (bias gradients). */
int stp_colsum(stp_ctx *ctx, int dtype, int32_t T, int32_t N, const void *x, float scale, float *out,
               int lane, void *hip_stream);
/* The same column sum for callers that cannot allocate device memory or supply a workspace (code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc): the stage-1 partials go to a fixed
 * 4 MiB array inside the library's device image instead of a workspace lane, so the call needs no
 * stp_set_workspace and performs no allocation.  Limit: ceil(T / 64) * N <= 1048576 (STP_ENOSPACE beyond it;
 * [6144, 4096] uses 393216).  Same kernels, same bits as stp_colsum.  Every call on one GPU shares that
 * GPU's array: calls that may overlap on one GPU (different streams) race; calls on one stream do not.
 * Nothing needs clearing between calls: the first kernel writes every partial the second one reads. */
int stp_colsum_noalloc(stp_ctx *ctx, int dtype, int32_t T, int32_t N, const void *x, float scale, float *out,
                       void *hip_stream);

/* Measurement aid: enqueues a one-wave kernel that spins for `milliseconds` of wall-clock time and
 * writes {shader-clock cycles elapsed, wall-clock ticks elapsed} to device_out2[0..1] (int64; the wall
 * clock ticks at hipDeviceAttributeWallClockRate kHz).  Run on a side stream while the units execute, it
 * yields the sustained shader clock the MFMA roofline should be read against. */
int stp_clock_probe(stp_ctx *ctx, long long *device_out2, double milliseconds, void *hip_stream);
/* The rate of that wall clock in kHz (hipDeviceAttributeWallClockRate of the context's device). */
int stp_wall_clock_khz(stp_ctx *ctx, int *khz);

#ifdef __cplusplus
}
#endif
#endif /* STP_H_ */

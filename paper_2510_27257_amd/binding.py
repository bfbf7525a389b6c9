"""ctypes declarations mirroring include/stp.h, plus small torch-side helpers that own
device memory (torch is used for allocation and streams only)."""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional, Sequence

__all__ = [
    "StpError", "lib", "lib_path", "LayerDesc", "Weights", "WGrads", "Stash", "Op", "Stage", "GemmArgs",
    "Context", "BOUNDARY_FN", "make_desc", "EXPORTED_SYMBOLS",
    "PRE_ATTN", "ATTN", "PRE_MLP", "MLP", "OP_F", "OP_B", "OP_W", "OP_BW", "F32", "BF16",
    "NORM_LN", "NORM_RMS", "ACT_GELU", "ACT_SWIGLU", "STASH_FIELDS", "STATUS",
    "OFFLOAD_W_ATTN", "OFFLOAD_W_MLP", "OFFLOAD_FWD", "offload_bytes",
    "ATTN_FWD", "ATTN_DKV", "ATTN_DQ", "attention_plan",
]

PRE_ATTN, ATTN, PRE_MLP, MLP = 0, 1, 2, 3
OP_F, OP_B, OP_W, OP_BW = 0, 1, 2, 3
F32, BF16 = 0, 1
NORM_LN, NORM_RMS = 0, 1
ACT_GELU, ACT_SWIGLU = 0, 1
OFFLOAD_W_ATTN, OFFLOAD_W_MLP, OFFLOAD_FWD = 0, 1, 2
STATUS = {0: "STP_OK", 1: "STP_EINVAL", 2: "STP_ESHAPE", 3: "STP_EALIGN", 4: "STP_ENOSPACE",
          5: "STP_ESEQ", 6: "STP_EUNSUPPORTED", 7: "STP_EHIP"}
STASH_FIELDS = ["X_LN", "STATS1", "QKV", "CTX", "LSE", "Z_LN", "STATS2", "H", "HU", "G", "DH", "DHU", "DG",
                "DQKV", "DCTX", "DELTA", "X_ATTN", "DX_ATTN", "DZ", "DX_LN"]

EXPORTED_SYMBOLS = [
    "stp_gemm_tile_hint", "stp_gemm_tile_hints_clear", "stp_create", "stp_destroy", "stp_last_error", "stp_status_str", "stp_check_desc", "stp_stash_bytes",
    "stp_stash_field", "stp_workspace_bytes", "stp_set_workspace", "stp_forward_unit",
    "stp_backward_input_unit", "stp_backward_weight_unit", "stp_braid_step", "stp_validate_ops",
    "stp_braid_reset", "stp_braid_detach", "stp_attention_plan", "stp_gemm", "stp_norm_forward", "stp_norm_backward", "stp_attention_forward",
    "stp_attention_backward", "stp_gelu_forward", "stp_gelu_backward", "stp_swiglu_forward",
    "stp_swiglu_backward", "stp_softmax_forward", "stp_softmax_backward", "stp_rope", "stp_colsum", "stp_colsum_noalloc", "stp_clock_probe", "stp_wall_clock_khz",
    "stp_offload_bytes", "stp_stash_offload", "stp_stash_reload",
]


class StpError(RuntimeError):
    def __init__(self, status: int, where: str, detail: str = ""):
        self.status = status
        super().__init__(f"{where}: {STATUS.get(status, status)} {detail}".strip())


class LayerDesc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("hidden", "heads_local", "head_dim", "ffn_local", "seq", "mbsz", "tp",
                                         "dtype", "norm", "act", "causal", "rope", "has_bias")] + \
               [("eps", C.c_float), ("rope_base", C.c_float), ("kv_heads_local", C.c_int32)]


_W_NAMES = ("norm1_g", "norm1_b", "w_qkv", "b_qkv", "w_o", "b_o", "norm2_g", "norm2_b", "w_fc1", "b_fc1",
            "w_up", "w_fc2", "b_fc2")


class Weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _W_NAMES]


class WGrads(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _W_NAMES]


class Stash(C.Structure):
    _fields_ = [("base", C.c_void_p), ("bytes", C.c_size_t)]


class Op(C.Structure):
    _fields_ = [("kind", C.c_int32), ("unit", C.c_int32), ("layer", C.c_int32), ("microbatch", C.c_int32)]


class Stage(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("n_microbatches", C.c_int32), ("desc", C.POINTER(LayerDesc)),
                ("w", C.POINTER(Weights)), ("g", C.POINTER(WGrads)), ("stash", C.POINTER(Stash)),
                ("act", C.POINTER(C.c_void_p)), ("grad", C.POINTER(C.c_void_p)),
                ("chain_break", C.POINTER(C.c_int32)),
                ("tail_act", C.POINTER(C.c_void_p)), ("tail_grad", C.POINTER(C.c_void_p))]


class GemmArgs(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("M", C.c_int32), ("N", C.c_int32), ("K", C.c_int32),
                ("A", C.c_void_p), ("lda", C.c_int32), ("a_trans", C.c_int32),
                ("B", C.c_void_p), ("ldb", C.c_int32), ("b_trans", C.c_int32),
                ("C", C.c_void_p), ("ldc", C.c_int32), ("c_f32_accum", C.c_int32),
                ("bias", C.c_void_p), ("bias_scale", C.c_float),
                ("resid", C.c_void_p), ("ldr", C.c_int32), ("resid_scale", C.c_float),
                ("epilogue", C.c_int32), ("C2", C.c_void_p), ("aux", C.c_void_p), ("ld2", C.c_int32),
                ("tile_m", C.c_int32), ("tile_n", C.c_int32)]


BOUNDARY_FN = C.CFUNCTYPE(None, C.c_void_p, C.c_int, C.c_void_p, C.c_size_t, C.c_int32, C.c_int32, C.c_void_p)


def lib_path() -> str:
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), "libstp.so")


_lib = None


def lib() -> C.CDLL:
    """Loads libstp.so (built in-tree).  Raises if it is missing: there is no fallback."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        raise FileNotFoundError(f"{path} not found: build it with `python -m paper_2510_27257_amd.build` "
                                "(or __graft_entry__.build())")
    L = C.CDLL(path)
    vp, i32, sz, f32 = C.c_void_p, C.c_int32, C.c_size_t, C.c_float
    P = C.POINTER
    L.stp_create.argtypes = [P(vp), C.c_int]
    L.stp_destroy.argtypes = [vp]
    L.stp_last_error.argtypes = [vp]
    L.stp_last_error.restype = C.c_char_p
    L.stp_status_str.argtypes = [C.c_int]
    L.stp_status_str.restype = C.c_char_p
    L.stp_check_desc.argtypes = [P(LayerDesc)]
    L.stp_stash_bytes.argtypes = [P(LayerDesc), P(sz)]
    L.stp_stash_field.argtypes = [P(LayerDesc), C.c_int, P(sz), P(sz)]
    L.stp_workspace_bytes.argtypes = [P(LayerDesc), P(sz)]
    L.stp_set_workspace.argtypes = [vp, vp, sz]
    L.stp_forward_unit.argtypes = [vp, P(LayerDesc), C.c_int, P(Weights), vp, vp, vp, P(Stash), C.c_int, vp]
    L.stp_backward_input_unit.argtypes = [vp, P(LayerDesc), C.c_int, P(Weights), P(Stash), vp, vp, vp, vp,
                                          P(WGrads), C.c_int, vp]
    L.stp_backward_weight_unit.argtypes = [vp, P(LayerDesc), C.c_int, P(Stash), vp, P(WGrads), C.c_int, vp]
    L.stp_braid_step.argtypes = [vp, P(Stage), P(Op), sz, vp, vp, vp, vp, vp]
    L.stp_validate_ops.argtypes = [P(Stage), P(Op), sz, P(sz)]
    L.stp_braid_reset.argtypes = [vp]
    L.stp_braid_detach.argtypes = [vp]
    L.stp_attention_plan.argtypes = [P(LayerDesc), C.c_int, P(i32), P(i32), P(i32), P(C.c_uint16), sz]
    L.stp_gemm.argtypes = [vp, P(GemmArgs), vp]
    L.stp_gemm_tile_hint.argtypes = [vp, i32, i32, i32, C.c_int, C.c_int, i32, i32]
    L.stp_gemm_tile_hints_clear.argtypes = [vp]
    L.stp_norm_forward.argtypes = [vp, C.c_int, C.c_int, i32, i32, f32, vp, vp, vp, vp, vp, vp]
    L.stp_norm_backward.argtypes = [vp, C.c_int, C.c_int, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, f32, C.c_int, vp]
    L.stp_attention_forward.argtypes = [vp, P(LayerDesc), vp, vp, vp, C.c_int, vp]
    L.stp_attention_backward.argtypes = [vp, P(LayerDesc), vp, vp, vp, vp, vp, vp, C.c_int, vp]
    L.stp_gelu_forward.argtypes = [vp, C.c_int, sz, vp, vp, vp]
    L.stp_gelu_backward.argtypes = [vp, C.c_int, sz, vp, vp, vp, vp]
    L.stp_swiglu_forward.argtypes = [vp, C.c_int, sz, vp, vp, vp, vp]
    L.stp_swiglu_backward.argtypes = [vp, C.c_int, sz, vp, vp, vp, vp, vp, vp]
    L.stp_softmax_forward.argtypes = [vp, C.c_int, i32, i32, f32, C.c_int, vp, vp, vp]
    L.stp_softmax_backward.argtypes = [vp, C.c_int, i32, i32, f32, vp, vp, vp, vp]
    L.stp_rope.argtypes = [vp, P(LayerDesc), vp, C.c_int, vp]
    L.stp_colsum.argtypes = [vp, C.c_int, i32, i32, vp, f32, vp, C.c_int, vp]
    L.stp_colsum_noalloc.argtypes = [vp, C.c_int, i32, i32, vp, f32, vp, vp]
    L.stp_clock_probe.argtypes = [vp, vp, C.c_double, vp]
    L.stp_wall_clock_khz.argtypes = [vp, P(C.c_int)]
    L.stp_offload_bytes.argtypes = [P(LayerDesc), C.c_int, f32, P(sz)]
    L.stp_stash_offload.argtypes = [vp, P(LayerDesc), C.c_int, f32, P(Stash), vp, sz, vp, vp]
    L.stp_stash_reload.argtypes = [vp, P(LayerDesc), C.c_int, f32, P(Stash), vp, sz, vp, vp]
    for name in EXPORTED_SYMBOLS:
        fn = getattr(L, name)
        if fn.restype is C.c_int or fn.restype is None or fn.restype == C.c_int:
            fn.restype = C.c_int
    L.stp_last_error.restype = C.c_char_p
    L.stp_status_str.restype = C.c_char_p
    _lib = L
    return L


def make_desc(wl, mbsz: int = 1, seq: Optional[int] = None) -> LayerDesc:
    """LayerDesc from a synth.Workload-like object (attribute names as in the header)."""
    return LayerDesc(hidden=wl.hidden, heads_local=wl.heads_local, head_dim=wl.head_dim, ffn_local=wl.ffn_local,
                     seq=wl.seq if seq is None else seq, mbsz=mbsz, tp=wl.tp,
                     dtype=BF16 if wl.dtype == "bf16" else F32,
                     norm=NORM_LN if wl.norm == "ln" else NORM_RMS,
                     act=ACT_GELU if wl.act == "gelu" else ACT_SWIGLU,
                     causal=int(wl.causal), rope=int(wl.rope), has_bias=int(wl.has_bias),
                     eps=wl.eps, rope_base=wl.rope_base, kv_heads_local=int(getattr(wl, "kv_heads", 0)))


def _ptr(t) -> Optional[int]:
    """Device address of a torch tensor (None passes NULL)."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(s) -> Optional[int]:
    if s is None:
        return None
    if isinstance(s, int):
        return s
    return s.cuda_stream


def offload_bytes(desc: "LayerDesc", which: int, alpha: float) -> int:
    """Host bytes stp_stash_offload moves for this layer, field set and fraction (no GPU needed)."""
    n = C.c_size_t()
    rc = lib().stp_offload_bytes(C.byref(desc), which, alpha, C.byref(n))
    if rc != 0:
        raise StpError(rc, "stp_offload_bytes")
    return n.value


ATTN_FWD, ATTN_DKV, ATTN_DQ = 0, 1, 2


def attention_plan(desc: "LayerDesc", kind: int):
    """(chunk_steps, max_chunks, [(block, chunk), ...] in dispatch order) of a chunked attention kernel (no GPU needed)."""
    cs, mc, n = C.c_int32(), C.c_int32(), C.c_int32()
    items = (C.c_uint16 * 1024)()
    rc = lib().stp_attention_plan(C.byref(desc), kind, C.byref(cs), C.byref(mc), C.byref(n), items, 1024)
    if rc != 0:
        raise StpError(rc, "stp_attention_plan")
    return cs.value, mc.value, [(items[i] & 0xfff, items[i] >> 12) for i in range(n.value)]


class Context:
    """Owns an stp_ctx and (optionally) a torch-allocated workspace for it."""

    def __init__(self, device: int = 0):
        self._lib = lib()
        self._h = C.c_void_p()
        st = self._lib.stp_create(C.byref(self._h), device)
        if st != 0:
            raise StpError(st, "stp_create", "(is a GPU present?)")
        self._ws = None
        self._keep = []

    def close(self):
        if self._h:
            self._lib.stp_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def handle(self):
        return self._h

    def check(self, status: int, where: str):
        if status != 0:
            raise StpError(status, where, self._lib.stp_last_error(self._h).decode())

    def last_error(self) -> str:
        return self._lib.stp_last_error(self._h).decode()

    # ---- sizes ---------------------------------------------------------------
    def stash_bytes(self, desc: LayerDesc) -> int:
        n = C.c_size_t()
        self.check(self._lib.stp_stash_bytes(C.byref(desc), C.byref(n)), "stp_stash_bytes")
        return n.value

    def stash_field(self, desc: LayerDesc, field) -> tuple:
        idx = STASH_FIELDS.index(field) if isinstance(field, str) else field
        off, n = C.c_size_t(), C.c_size_t()
        self.check(self._lib.stp_stash_field(C.byref(desc), idx, C.byref(off), C.byref(n)), "stp_stash_field")
        return off.value, n.value

    def workspace_bytes(self, desc: LayerDesc) -> int:
        n = C.c_size_t()
        self.check(self._lib.stp_workspace_bytes(C.byref(desc), C.byref(n)), "stp_workspace_bytes")
        return n.value

    def set_workspace(self, tensor):
        self._ws = tensor
        self.check(self._lib.stp_set_workspace(self._h, _ptr(tensor), tensor.numel() * tensor.element_size()
                                               if tensor is not None else 0), "stp_set_workspace")

    def ensure_workspace(self, descs: Sequence[LayerDesc]):
        import torch
        need = max(self.workspace_bytes(d) for d in descs)
        if self._ws is None or self._ws.numel() < need:
            # kernels already enqueued on any stream may still use the old block (and its lane offsets)
            torch.cuda.synchronize()
            self.set_workspace(torch.empty(need, dtype=torch.uint8, device="cuda"))

    # ---- units ---------------------------------------------------------------
    def forward_unit(self, desc, unit, w: Weights, stash: Stash, x_in=None, x_resid=None, y_out=None, lane=0,
                     stream=None):
        self.check(self._lib.stp_forward_unit(self._h, C.byref(desc), unit, C.byref(w), _ptr(x_in), _ptr(x_resid),
                                              _ptr(y_out), C.byref(stash), lane, _stream(stream)),
                   "stp_forward_unit")

    def backward_input_unit(self, desc, unit, w: Weights, stash: Stash, dy, dx, x_in=None, d_resid=None,
                            wgrads: Optional[WGrads] = None, lane=0, stream=None):
        self.check(self._lib.stp_backward_input_unit(self._h, C.byref(desc), unit, C.byref(w), C.byref(stash),
                                                     _ptr(x_in), _ptr(dy), _ptr(d_resid), _ptr(dx),
                                                     C.byref(wgrads) if wgrads is not None else None, lane,
                                                     _stream(stream)), "stp_backward_input_unit")

    def backward_weight_unit(self, desc, unit, stash: Stash, dy, wgrads: WGrads, lane=0, stream=None):
        self.check(self._lib.stp_backward_weight_unit(self._h, C.byref(desc), unit, C.byref(stash), _ptr(dy),
                                                      C.byref(wgrads), lane, _stream(stream)),
                   "stp_backward_weight_unit")

    def braid_step(self, stage: Stage, ops, s_fwd, s_bwd, s_wgrad, cb=None, user=None):
        arr = ops if isinstance(ops, C.Array) else (Op * len(ops))(*ops)
        cbp = C.cast(cb, C.c_void_p) if cb is not None else None
        self.check(self._lib.stp_braid_step(self._h, C.byref(stage), arr, len(arr), _stream(s_fwd), _stream(s_bwd),
                                            _stream(s_wgrad), cbp, user), "stp_braid_step")

    def braid_reset(self):
        self.check(self._lib.stp_braid_reset(self._h), "stp_braid_reset")

    def braid_detach(self):
        self.check(self._lib.stp_braid_detach(self._h), "stp_braid_detach")

    # ---- kernels -------------------------------------------------------------
    def gemm(self, args: GemmArgs, stream=None):
        self.check(self._lib.stp_gemm(self._h, C.byref(args), _stream(stream)), "stp_gemm")

    def gemm_tile_hint(self, M, N, K, a_trans, b_trans, tile_m, tile_n):
        self.check(self._lib.stp_gemm_tile_hint(self._h, M, N, K, int(a_trans), int(b_trans), tile_m, tile_n),
                   "stp_gemm_tile_hint")

    def gemm_tile_hints_clear(self):
        self.check(self._lib.stp_gemm_tile_hints_clear(self._h), "stp_gemm_tile_hints_clear")

    def norm_forward(self, dtype, norm, T, h, eps, x, gamma, beta, y, stats, stream=None):
        self.check(self._lib.stp_norm_forward(self._h, dtype, norm, T, h, eps, _ptr(x), _ptr(gamma), _ptr(beta),
                                              _ptr(y), _ptr(stats), _stream(stream)), "stp_norm_forward")

    def norm_backward(self, dtype, norm, T, h, x, gamma, stats, dy, d_resid, dx, dgamma, dbeta, lane=0, stream=None,
                      d_resid_sum=None, d_resid_sum_scale=1.0):
        self.check(self._lib.stp_norm_backward(self._h, dtype, norm, T, h, _ptr(x), _ptr(gamma), _ptr(stats),
                                               _ptr(dy), _ptr(d_resid), _ptr(dx), _ptr(dgamma), _ptr(dbeta),
                                               _ptr(d_resid_sum), d_resid_sum_scale, lane,
                                               _stream(stream)), "stp_norm_backward")

    def attention_forward(self, desc, qkv, out, lse, lane=0, stream=None):
        self.check(self._lib.stp_attention_forward(self._h, C.byref(desc), _ptr(qkv), _ptr(out), _ptr(lse), lane,
                                                   _stream(stream)), "stp_attention_forward")

    def attention_backward(self, desc, qkv, out, lse, dout, delta, dqkv, lane=0, stream=None):
        self.check(self._lib.stp_attention_backward(self._h, C.byref(desc), _ptr(qkv), _ptr(out), _ptr(lse),
                                                    _ptr(dout), _ptr(delta), _ptr(dqkv), lane, _stream(stream)),
                   "stp_attention_backward")

    def gelu_forward(self, dtype, n, x, y, stream=None):
        self.check(self._lib.stp_gelu_forward(self._h, dtype, n, _ptr(x), _ptr(y), _stream(stream)),
                   "stp_gelu_forward")

    def gelu_backward(self, dtype, n, x, dy, dx, stream=None):
        self.check(self._lib.stp_gelu_backward(self._h, dtype, n, _ptr(x), _ptr(dy), _ptr(dx), _stream(stream)),
                   "stp_gelu_backward")

    def swiglu_forward(self, dtype, n, gate, up, y, stream=None):
        self.check(self._lib.stp_swiglu_forward(self._h, dtype, n, _ptr(gate), _ptr(up), _ptr(y), _stream(stream)),
                   "stp_swiglu_forward")

    def swiglu_backward(self, dtype, n, gate, up, dy, dgate, dup, stream=None):
        self.check(self._lib.stp_swiglu_backward(self._h, dtype, n, _ptr(gate), _ptr(up), _ptr(dy), _ptr(dgate),
                                                 _ptr(dup), _stream(stream)), "stp_swiglu_backward")

    def softmax_forward(self, dtype, rows, n, scale, causal, x, y, stream=None):
        self.check(self._lib.stp_softmax_forward(self._h, dtype, rows, n, scale, int(causal), _ptr(x), _ptr(y),
                                                 _stream(stream)), "stp_softmax_forward")

    def softmax_backward(self, dtype, rows, n, scale, y, dy, dx, stream=None):
        self.check(self._lib.stp_softmax_backward(self._h, dtype, rows, n, scale, _ptr(y), _ptr(dy), _ptr(dx),
                                                  _stream(stream)), "stp_softmax_backward")

    def rope(self, desc, qkv, inverse=False, stream=None):
        self.check(self._lib.stp_rope(self._h, C.byref(desc), _ptr(qkv), int(inverse), _stream(stream)), "stp_rope")

    def stash_offload(self, desc, which, alpha, stash, host, s_producer, s_copy):
        """host: page-locked CPU uint8 tensor of at least offload_bytes(desc, which, alpha) bytes."""
        self.check(self._lib.stp_stash_offload(self._h, C.byref(desc), which, alpha, C.byref(stash), host.data_ptr(),
                                               host.numel() * host.element_size(), _stream(s_producer), _stream(s_copy)),
                   "stp_stash_offload")

    def stash_reload(self, desc, which, alpha, stash, host, s_copy, s_consumer):
        self.check(self._lib.stp_stash_reload(self._h, C.byref(desc), which, alpha, C.byref(stash), host.data_ptr(),
                                              host.numel() * host.element_size(), _stream(s_copy), _stream(s_consumer)),
                   "stp_stash_reload")

    def clock_probe(self, out2, milliseconds, stream=None):
        """out2: int64 device tensor with 2 elements -> (shader cycles, wall ticks at 100 MHz-class rate)."""
        self.check(self._lib.stp_clock_probe(self._h, _ptr(out2), float(milliseconds), _stream(stream)),
                   "stp_clock_probe")

    def wall_clock_khz(self) -> int:
        """Rate of the constant wall clock the clock probe reads, in kHz."""
        k = C.c_int()
        self.check(self._lib.stp_wall_clock_khz(self._h, C.byref(k)), "stp_wall_clock_khz")
        return k.value

    def colsum(self, dtype, T, N, x, scale, out, lane=0, stream=None):
        self.check(self._lib.stp_colsum(self._h, dtype, T, N, _ptr(x), scale, _ptr(out), lane, _stream(stream)),
                   "stp_colsum")

    def colsum_noalloc(self, dtype, T, N, x, scale, out, stream=None):
        """stp_colsum with its partial sums in the library's fixed scratch array: no workspace, no allocation."""
        self.check(self._lib.stp_colsum_noalloc(self._h, dtype, T, N, _ptr(x), scale, _ptr(out), _stream(stream)),
                   "stp_colsum_noalloc")

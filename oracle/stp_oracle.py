"""CPU fp64 oracle for the fine-grained computation units of one TP shard.

THIS IS TEST INFRASTRUCTURE, NOT PART OF THE PRODUCT.  Only the test-suite, the
smoke entry and the benchmark's cpu_baseline leg may import it.  It shares no
code with the HIP path: every formula below is the plain definition, evaluated
in numpy float64 with library matmul / exp / erf as the only primitives, no
blocking, no fusion, no re-ordering.

What it computes (paper Section 3):
  * a pre-norm transformer layer is cut into four units, Pre-Attn, Attn,
    Pre-MLP, MLP (Section 3, second paragraph);
  * the residual add is folded into the Attn / MLP unit *before* the TP
    reduction: each of the t ranks adds detach(X)/t to its partial (Eq. 1);
  * in backward the residual contributes an un-reduced "+1" path (Eq. 2);
  * Attn and MLP backward are split, after Zero Bubble, into an activation
    gradient part (B) and a weight gradient part (W) (Section 3).

Readings taken where the paper is silent are listed next to each function and
collected in the repository's design notes (norm epsilon, exact-erf GELU,
[Q|K|V] head-major column order, rotate-half RoPE, b/t bias on row-parallel
linears, norm gain/bias gradients produced by the Pre-* backward units).

Parity pins (tests/test_oracle_*.py): torch-autograd fp64 of a textbook layer
built from library routines, central finite differences, brute-force scalar
loops, closed forms, TP-sum invariants of Eq. 1-2, B+W == fused backward.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Optional

import numpy as np
from scipy.special import erf as _erf

PRE_ATTN, ATTN, PRE_MLP, MLP = 0, 1, 2, 3
UNIT_NAMES = ("pre_attn", "attn", "pre_mlp", "mlp")


@dataclass(frozen=True)
class LayerCfg:
    hidden: int          # h
    heads_local: int     # n  (heads held by this rank)
    head_dim: int        # d
    ffn_local: int       # f  (FFN columns held by this rank)
    tp: int = 1          # t
    norm: str = "ln"     # "ln" | "rms"
    act: str = "gelu"    # "gelu" | "swiglu"
    causal: bool = True
    rope: bool = False
    has_bias: bool = True
    eps: float = 1e-5
    rope_base: float = 10000.0
    kv_heads_local: int = 0   # key / value heads held by this rank; 0 = one per query head (the model table of
                              # Section 5.1 lists 40 / 8 and 56 / 8 query / key-value heads: grouped-query attention)

    @property
    def attn_local(self) -> int:
        return self.heads_local * self.head_dim

    @property
    def kv_heads(self) -> int:
        return self.kv_heads_local or self.heads_local

    @property
    def kv_local(self) -> int:
        return self.kv_heads * self.head_dim


# --------------------------------------------------------------------------
# Normalisation (Pre-Attn / Pre-MLP units; Eq. 1, X_ln = LayerNorm(X))
# --------------------------------------------------------------------------
def norm_fwd(cfg: LayerCfg, X, gamma, beta=None):
    """LayerNorm (biased variance) or RMSNorm over the last axis."""
    X = np.asarray(X, np.float64)
    if cfg.norm == "ln":
        mu = X.mean(axis=1, keepdims=True)
        var = ((X - mu) ** 2).mean(axis=1, keepdims=True)
        xhat = (X - mu) / np.sqrt(var + cfg.eps)
        Y = xhat * gamma
        if beta is not None:
            Y = Y + beta
        return Y
    ms = (X ** 2).mean(axis=1, keepdims=True)
    return X / np.sqrt(ms + cfg.eps) * gamma


def norm_bwd(cfg: LayerCfg, dY, X, gamma):
    """Gradient of norm_fwd w.r.t. X, gamma and beta (beta grad is None for RMSNorm)."""
    X = np.asarray(X, np.float64)
    dY = np.asarray(dY, np.float64)
    h = X.shape[1]
    if cfg.norm == "ln":
        mu = X.mean(axis=1, keepdims=True)
        var = ((X - mu) ** 2).mean(axis=1, keepdims=True)
        rstd = 1.0 / np.sqrt(var + cfg.eps)
        xhat = (X - mu) * rstd
        g = dY * gamma
        dX = rstd * (g - g.mean(axis=1, keepdims=True)
                     - xhat * (g * xhat).mean(axis=1, keepdims=True))
        return dX, (dY * xhat).sum(axis=0), dY.sum(axis=0)
    ms = (X ** 2).mean(axis=1, keepdims=True)
    r = 1.0 / np.sqrt(ms + cfg.eps)
    g = dY * gamma
    dX = r * g - X * (r ** 3) * (g * X).sum(axis=1, keepdims=True) / h
    return dX, (dY * X * r).sum(axis=0), None


# --------------------------------------------------------------------------
# Activations (MLP unit)
# --------------------------------------------------------------------------
def gelu(x):
    """Exact GELU, x * Phi(x)."""
    return 0.5 * x * (1.0 + _erf(x / np.sqrt(2.0)))


def gelu_grad(x):
    """d/dx [x Phi(x)] = Phi(x) + x phi(x)."""
    Phi = 0.5 * (1.0 + _erf(x / np.sqrt(2.0)))
    phi = np.exp(-0.5 * x * x) / np.sqrt(2.0 * np.pi)
    return Phi + x * phi


def silu(x):
    return x / (1.0 + np.exp(-x))


def silu_grad(x):
    sg = 1.0 / (1.0 + np.exp(-x))
    return sg * (1.0 + x * (1.0 - sg))


# --------------------------------------------------------------------------
# Rotary position embedding (rotate-half pairing (i, i + d/2), positions 0..s-1)
# --------------------------------------------------------------------------
def rope(x, base: float, inverse: bool = False):
    """x: [s, n, d].  Rotates pair (x_i, x_{i+d/2}) of token p by angle p*base^(-2i/d).

    inverse=True applies the transpose rotation (used on gradients)."""
    s, n, d = x.shape
    half = d // 2
    inv_freq = base ** (-2.0 * np.arange(half, dtype=np.float64) / d)
    ang = np.arange(s, dtype=np.float64)[:, None] * inv_freq[None, :]     # [s, half]
    c, sn = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    if inverse:
        sn = -sn
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * sn, x2 * c + x1 * sn], axis=-1)


# --------------------------------------------------------------------------
# Row softmax on its own (the normalisation inside "Attention(.)" of Eq. 1, as a stand-alone operation:
# the HIP side has a stand-alone softmax kernel pair that is judged on memory bandwidth)
# --------------------------------------------------------------------------
def softmax_fwd(x, scale: float = 1.0, causal: bool = False):
    """y[r, :] = softmax(scale * x[r, :]).  causal: the rows are stacked [n, n] squares and element j of row r is
    masked when j > r mod n (a key after the query)."""
    x = np.asarray(x, np.float64) * scale
    rows, n = x.shape
    if causal:
        r = np.arange(rows)[:, None] % n
        x = np.where(np.arange(n)[None, :] <= r, x, -np.inf)
    e = np.exp(x - x.max(axis=1, keepdims=True))
    return e / e.sum(axis=1, keepdims=True)


def softmax_bwd(y, dy, scale: float = 1.0):
    """Gradient w.r.t. x of softmax_fwd given its output y and the upstream gradient dy:
    dx = scale * y o (dy - rowsum(dy o y))."""
    y, dy = np.asarray(y, np.float64), np.asarray(dy, np.float64)
    return scale * y * (dy - (dy * y).sum(axis=1, keepdims=True))


# --------------------------------------------------------------------------
# Attention core (per head, no communication; "Attention(.)" of Eq. 1)
# --------------------------------------------------------------------------
def _probs(q, k, causal: bool):
    """softmax_rows(q k^T / sqrt(d)) with optional causal mask (key j > query i masked)."""
    s, d = q.shape
    S = (q @ k.T) / np.sqrt(d)
    if causal:
        S = np.where(np.tril(np.ones((s, k.shape[0]), dtype=bool)), S, -np.inf)
    S = S - S.max(axis=1, keepdims=True)
    E = np.exp(S)
    return E / E.sum(axis=1, keepdims=True)


def attention_fwd(q, k, v, causal: bool):
    """q: [s, n, d]; k, v: [s, n_kv, d] with n a multiple of n_kv -> ctx [s, n, d].

    Query head i attends to key / value head i // (n / n_kv) (grouped-query attention; n_kv = n is the
    ordinary multi-head case)."""
    out = np.empty_like(q)
    group = q.shape[1] // k.shape[1]
    for hd in range(q.shape[1]):
        out[:, hd, :] = _probs(q[:, hd, :], k[:, hd // group, :], causal) @ v[:, hd // group, :]
    return out


def attention_bwd(q, k, v, dctx, causal: bool):
    """Gradients of attention_fwd w.r.t. q, k, v."""
    dq, dk, dv = np.empty_like(q), np.zeros_like(k), np.zeros_like(v)
    d = q.shape[2]
    group = q.shape[1] // k.shape[1]
    for hd in range(q.shape[1]):
        kh = hd // group                      # a key / value head collects the gradients of its whole group
        P = _probs(q[:, hd, :], k[:, kh, :], causal)
        do = dctx[:, hd, :]
        dv[:, kh, :] += P.T @ do
        dP = do @ v[:, kh, :].T
        dS = P * (dP - (dP * P).sum(axis=1, keepdims=True))
        dq[:, hd, :] = dS @ k[:, kh, :] / np.sqrt(d)
        dk[:, kh, :] += dS.T @ q[:, hd, :] / np.sqrt(d)
    return dq, dk, dv


# --------------------------------------------------------------------------
# The four forward units of one TP rank (Section 3; Eq. 1)
# --------------------------------------------------------------------------
def forward_unit(cfg: LayerCfg, unit: int, w: Dict[str, np.ndarray], stash: dict,
                 x_in=None, x_resid=None):
    """Runs one forward unit of one rank.  `stash` collects what B and W need.

    PRE_ATTN: x_in = X            -> returns X_ln
    ATTN    : x_resid = X         -> returns this rank's partial of X_attn (before AR)
    PRE_MLP : x_in = X_attn       -> returns Z_ln
    MLP     : x_resid = X_attn    -> returns this rank's partial of the layer output
    """
    t = cfg.tp
    n, d, a = cfg.heads_local, cfg.head_dim, cfg.attn_local
    if unit == PRE_ATTN:
        stash["x"] = np.asarray(x_in, np.float64)
        stash["x_ln"] = norm_fwd(cfg, stash["x"], w["norm1_g"], w.get("norm1_b"))
        return stash["x_ln"]
    if unit == ATTN:
        s = stash["x_ln"].shape[0]
        qkv = stash["x_ln"] @ w["w_qkv"]
        if cfg.has_bias:
            qkv = qkv + w["b_qkv"]
        nk, ak = cfg.kv_heads, cfg.kv_local       # columns of QKV: [Q heads | K heads | V heads]
        q = qkv[:, :a].reshape(s, n, d)
        k = qkv[:, a:a + ak].reshape(s, nk, d)
        v = qkv[:, a + ak:a + 2 * ak].reshape(s, nk, d)
        if cfg.rope:
            q, k = rope(q, cfg.rope_base), rope(k, cfg.rope_base)
        ctx = attention_fwd(q, k, v, cfg.causal).reshape(s, a)
        stash.update(q=q, k=k, v=v, ctx=ctx)
        y = ctx @ w["w_o"] + np.asarray(x_resid, np.float64) / t      # Eq. 1: + detach(X)/t
        if cfg.has_bias:
            y = y + w["b_o"] / t
        return y
    if unit == PRE_MLP:
        stash["x_attn"] = np.asarray(x_in, np.float64)
        stash["z_ln"] = norm_fwd(cfg, stash["x_attn"], w["norm2_g"], w.get("norm2_b"))
        return stash["z_ln"]
    if unit == MLP:
        z = stash["z_ln"]
        if cfg.act == "gelu":
            hpre = z @ w["w_fc1"]
            if cfg.has_bias:
                hpre = hpre + w["b_fc1"]
            g = gelu(hpre)
            stash.update(h=hpre, g=g)
        else:
            hg, hu = z @ w["w_fc1"], z @ w["w_up"]
            if cfg.has_bias:
                hg = hg + w["b_fc1"]
            g = silu(hg) * hu
            stash.update(h=hg, hu=hu, g=g)
        o = g @ w["w_fc2"] + np.asarray(x_resid, np.float64) / t
        if cfg.has_bias:
            o = o + w["b_fc2"] / t
        return o
    raise ValueError(unit)


# --------------------------------------------------------------------------
# B units: activation gradients (Section 3; Eq. 2)
# --------------------------------------------------------------------------
def backward_input_unit(cfg: LayerCfg, unit: int, w, stash: dict, dy, d_resid=None,
                        grads: Optional[dict] = None):
    """One activation-gradient unit of one rank.

    MLP     : dy = dX_out            -> this rank's partial of dZ_ln (before AR); stashes dH
    PRE_MLP : dy = dZ_ln (reduced), d_resid = dX_out -> dX_attn  (Eq. 2's "+1" path)
    ATTN    : dy = dX_attn           -> this rank's partial of dX_ln; stashes dQKV
    PRE_ATTN: dy = dX_ln (reduced), d_resid = dX_attn -> dX
    Norm gain / bias gradients are accumulated into `grads` by the PRE_* units.
    """
    n, d, a = cfg.heads_local, cfg.head_dim, cfg.attn_local
    dy = np.asarray(dy, np.float64)
    if unit == MLP:
        dg = dy @ w["w_fc2"].T
        if cfg.act == "gelu":
            dh = dg * gelu_grad(stash["h"])
            stash["dh"] = dh
            return dh @ w["w_fc1"].T
        dhg = dg * stash["hu"] * silu_grad(stash["h"])
        dhu = dg * silu(stash["h"])
        stash.update(dh=dhg, dhu=dhu)
        return dhg @ w["w_fc1"].T + dhu @ w["w_up"].T
    if unit in (PRE_MLP, PRE_ATTN):
        x = stash["x_attn"] if unit == PRE_MLP else stash["x"]
        pre = "norm2" if unit == PRE_MLP else "norm1"
        dx, dgam, dbet = norm_bwd(cfg, dy, x, w[pre + "_g"])
        if grads is not None:
            _acc(grads, pre + "_g", dgam)
            if dbet is not None and (pre + "_b") in w:
                _acc(grads, pre + "_b", dbet)
        return dx + np.asarray(d_resid, np.float64)                  # Eq. 2: "+1"
    if unit == ATTN:
        s = dy.shape[0]
        dctx = (dy @ w["w_o"].T).reshape(s, n, d)
        dq, dk, dv = attention_bwd(stash["q"], stash["k"], stash["v"], dctx, cfg.causal)
        if cfg.rope:
            dq, dk = rope(dq, cfg.rope_base, inverse=True), rope(dk, cfg.rope_base, inverse=True)
        dqkv = np.concatenate([dq.reshape(s, a), dk.reshape(s, cfg.kv_local), dv.reshape(s, cfg.kv_local)], axis=1)
        stash["dqkv"] = dqkv
        return dqkv @ w["w_qkv"].T
    raise ValueError(unit)


# --------------------------------------------------------------------------
# W units: weight gradients (Section 3, split after Zero Bubble)
# --------------------------------------------------------------------------
def _acc(grads: dict, key: str, val):
    grads[key] = grads[key] + val if key in grads else np.array(val, np.float64)


def backward_weight_unit(cfg: LayerCfg, unit: int, stash: dict, dy, grads: dict):
    """MLP: dy = dX_out.  ATTN: dy = dX_attn.  Accumulates into `grads`."""
    dy = np.asarray(dy, np.float64)
    t = cfg.tp
    if unit == MLP:
        _acc(grads, "w_fc2", stash["g"].T @ dy)
        _acc(grads, "w_fc1", stash["z_ln"].T @ stash["dh"])
        if cfg.act == "swiglu":
            _acc(grads, "w_up", stash["z_ln"].T @ stash["dhu"])
        if cfg.has_bias:
            _acc(grads, "b_fc1", stash["dh"].sum(axis=0))
            _acc(grads, "b_fc2", dy.sum(axis=0) / t)
        return
    if unit == ATTN:
        _acc(grads, "w_o", stash["ctx"].T @ dy)
        _acc(grads, "w_qkv", stash["x_ln"].T @ stash["dqkv"])
        if cfg.has_bias:
            _acc(grads, "b_qkv", stash["dqkv"].sum(axis=0))
            _acc(grads, "b_o", dy.sum(axis=0) / t)
        return
    raise ValueError(unit)


# --------------------------------------------------------------------------
# Whole-layer drivers used by the tests (all ranks, reductions at the boundaries)
# --------------------------------------------------------------------------
def layer_forward_all_ranks(cfg: LayerCfg, shards, X):
    """Runs the 4 forward units on every rank, summing partials where Eq. 1 has AR."""
    stashes = [dict() for _ in shards]
    for w, st in zip(shards, stashes):
        forward_unit(cfg, PRE_ATTN, w, st, x_in=X)
    x_attn = sum(forward_unit(cfg, ATTN, w, st, x_resid=X) for w, st in zip(shards, stashes))
    for w, st in zip(shards, stashes):
        forward_unit(cfg, PRE_MLP, w, st, x_in=x_attn)
    x_out = sum(forward_unit(cfg, MLP, w, st, x_resid=x_attn) for w, st in zip(shards, stashes))
    return x_out, stashes


def layer_backward_all_ranks(cfg: LayerCfg, shards, stashes, dX_out):
    """B then W units on every rank; returns dX and the per-rank gradient dicts."""
    grads = [dict() for _ in shards]
    dz = sum(backward_input_unit(cfg, MLP, w, st, dX_out) for w, st in zip(shards, stashes))
    dxa = None
    for w, st, g in zip(shards, stashes, grads):
        dxa = backward_input_unit(cfg, PRE_MLP, w, st, dz, d_resid=dX_out, grads=g)
    dxl = sum(backward_input_unit(cfg, ATTN, w, st, dxa) for w, st in zip(shards, stashes))
    dx = None
    for w, st, g in zip(shards, stashes, grads):
        dx = backward_input_unit(cfg, PRE_ATTN, w, st, dxl, d_resid=dxa, grads=g)
    for st, g in zip(stashes, grads):
        backward_weight_unit(cfg, MLP, st, dX_out, g)
        backward_weight_unit(cfg, ATTN, st, dxa, g)
    return dx, grads


def shard_weights(cfg_full: LayerCfg, W: Dict[str, np.ndarray], t: int, r: int):
    """Megatron-style split of an unsharded layer's weights for rank r of t.

    QKV and FC1 (and the SwiGLU up-projection) are split by output column, whole
    heads per rank, keeping the [Q | K | V] head-major order inside each rank;
    the out-projection and FC2 are split by input row; norm parameters and the
    row-parallel biases are replicated.
    """
    n, d = cfg_full.heads_local, cfg_full.head_dim
    a, f = n * d, cfg_full.ffn_local
    al, fl = a // t, f // t
    nk, ak = cfg_full.kv_heads, cfg_full.kv_local
    akl = ak // t                              # whole key / value heads per rank: n_kv must be a multiple of t
    out = {}
    for key in ("norm1_g", "norm1_b", "norm2_g", "norm2_b", "b_o", "b_fc2"):
        if key in W:
            out[key] = W[key]
    cols = np.concatenate([np.arange(r * al, (r + 1) * al),
                           np.arange(a + r * akl, a + (r + 1) * akl),
                           np.arange(a + ak + r * akl, a + ak + (r + 1) * akl)])
    out["w_qkv"] = W["w_qkv"][:, cols]
    if "b_qkv" in W:
        out["b_qkv"] = W["b_qkv"][cols]
    out["w_o"] = W["w_o"][r * al:(r + 1) * al, :]
    out["w_fc1"] = W["w_fc1"][:, r * fl:(r + 1) * fl]
    if "b_fc1" in W:
        out["b_fc1"] = W["b_fc1"][r * fl:(r + 1) * fl]
    if "w_up" in W:
        out["w_up"] = W["w_up"][:, r * fl:(r + 1) * fl]
    out["w_fc2"] = W["w_fc2"][r * fl:(r + 1) * fl, :]
    cfg_r = replace(cfg_full, heads_local=n // t, ffn_local=fl, tp=t,
                    kv_heads_local=(nk // t if cfg_full.kv_heads_local else 0))
    return cfg_r, out


# --------------------------------------------------------------------------
# Independently written fused full backward (no B/W split), used to check that
# B-units plus W-units together equal an ordinary backward pass.
# --------------------------------------------------------------------------
def fused_layer_backward(cfg: LayerCfg, w, X, dX_out, reduce_fn=None):
    """Single reverse sweep of one rank's layer producing dX and all weight grads.

    Written separately from the unit functions: it recomputes the forward
    from X, then walks backwards accumulating input and weight gradients
    together, operator by operator.  `reduce_fn(name, partial)` models the AR
    points (identity when None).
    """
    red = reduce_fn if reduce_fn is not None else (lambda name, v: v)
    t, n, d, a = cfg.tp, cfg.heads_local, cfg.head_dim, cfg.attn_local
    X = np.asarray(X, np.float64)
    s = X.shape[0]
    G: Dict[str, np.ndarray] = {}
    # ---- forward, keeping everything ----
    x_ln = norm_fwd(cfg, X, w["norm1_g"], w.get("norm1_b"))
    qkv = x_ln @ w["w_qkv"] + (w["b_qkv"] if cfg.has_bias else 0.0)
    nk, ak = cfg.kv_heads, cfg.kv_local
    q = qkv[:, :a].reshape(s, n, d)
    k, v = (qkv[:, a + i * ak:a + (i + 1) * ak].reshape(s, nk, d) for i in range(2))
    if cfg.rope:
        q, k = rope(q, cfg.rope_base), rope(k, cfg.rope_base)
    ctx = attention_fwd(q, k, v, cfg.causal).reshape(s, a)
    y = ctx @ w["w_o"] + X / t + (w["b_o"] / t if cfg.has_bias else 0.0)
    x_attn = red("x_attn", y)
    z_ln = norm_fwd(cfg, x_attn, w["norm2_g"], w.get("norm2_b"))
    h1 = z_ln @ w["w_fc1"] + (w["b_fc1"] if cfg.has_bias else 0.0)
    if cfg.act == "gelu":
        g = gelu(h1)
    else:
        hu = z_ln @ w["w_up"]
        g = silu(h1) * hu
    # ---- reverse sweep ----
    dO = np.asarray(dX_out, np.float64)
    G["w_fc2"] = np.einsum("sf,sh->fh", g, dO)
    if cfg.has_bias:
        G["b_fc2"] = dO.sum(0) / t
    dg = np.einsum("sh,fh->sf", dO, w["w_fc2"])
    if cfg.act == "gelu":
        dh1 = dg * gelu_grad(h1)
        dz = np.einsum("sf,hf->sh", dh1, w["w_fc1"])
    else:
        dh1 = dg * hu * silu_grad(h1)
        dhu = dg * silu(h1)
        G["w_up"] = np.einsum("sh,sf->hf", z_ln, dhu)
        dz = np.einsum("sf,hf->sh", dh1, w["w_fc1"]) + np.einsum("sf,hf->sh", dhu, w["w_up"])
    G["w_fc1"] = np.einsum("sh,sf->hf", z_ln, dh1)
    if cfg.has_bias:
        G["b_fc1"] = dh1.sum(0)
    dz = red("dz", dz)
    dxa_n, G["norm2_g"], b2 = norm_bwd(cfg, dz, x_attn, w["norm2_g"])
    if b2 is not None and "norm2_b" in w:
        G["norm2_b"] = b2
    dxa = dxa_n + dO
    G["w_o"] = np.einsum("sa,sh->ah", ctx, dxa)
    if cfg.has_bias:
        G["b_o"] = dxa.sum(0) / t
    dctx = np.einsum("sh,ah->sa", dxa, w["w_o"]).reshape(s, n, d)
    dq, dk, dv = attention_bwd(q, k, v, dctx, cfg.causal)
    if cfg.rope:
        dq, dk = rope(dq, cfg.rope_base, True), rope(dk, cfg.rope_base, True)
    dqkv = np.concatenate([dq.reshape(s, a), dk.reshape(s, ak), dv.reshape(s, ak)], 1)
    G["w_qkv"] = np.einsum("sh,sc->hc", x_ln, dqkv)
    if cfg.has_bias:
        G["b_qkv"] = dqkv.sum(0)
    dxl = red("dx_ln", np.einsum("sc,hc->sh", dqkv, w["w_qkv"]))
    dx_n, G["norm1_g"], b1 = norm_bwd(cfg, dxl, X, w["norm1_g"])
    if b1 is not None and "norm1_b" in w:
        G["norm1_b"] = b1
    return dx_n + dxa, G

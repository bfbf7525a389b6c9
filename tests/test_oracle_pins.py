"""CPU-only pins of the fp64 oracle against things other than itself.

Each test is chosen so that a plausible slip in oracle/stp_oracle.py (dropped
term, wrong sign, transposed operand, wrong 1/t factor) fails at least one.
"""
import math
import os
from dataclasses import replace

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import stp_oracle as O

HERE = os.path.dirname(os.path.abspath(__file__))


def rand_weights(cfg, rng, scale=0.3):
    h, a, f = cfg.hidden, cfg.attn_local, cfg.ffn_local
    c = a + 2 * cfg.kv_local
    W = {"norm1_g": 1 + 0.2 * rng.standard_normal(h), "norm2_g": 1 + 0.2 * rng.standard_normal(h),
         "w_qkv": scale * rng.standard_normal((h, c)), "w_o": scale * rng.standard_normal((a, h)),
         "w_fc1": scale * rng.standard_normal((h, f)), "w_fc2": scale * rng.standard_normal((f, h))}
    if cfg.norm == "ln":
        W["norm1_b"] = 0.2 * rng.standard_normal(h)
        W["norm2_b"] = 0.2 * rng.standard_normal(h)
    if cfg.act == "swiglu":
        W["w_up"] = scale * rng.standard_normal((h, f))
    if cfg.has_bias:
        W.update(b_qkv=0.2 * rng.standard_normal(c), b_o=0.2 * rng.standard_normal(h),
                 b_fc1=0.2 * rng.standard_normal(f), b_fc2=0.2 * rng.standard_normal(h))
    return W


VARIANTS = [
    dict(norm="ln", act="gelu", causal=True, rope=False, has_bias=True),
    dict(norm="rms", act="swiglu", causal=True, rope=True, has_bias=False),
    dict(norm="ln", act="gelu", causal=False, rope=False, has_bias=True),
    dict(norm="rms", act="gelu", causal=False, rope=True, has_bias=True),
    dict(norm="ln", act="swiglu", causal=True, rope=True, has_bias=True),
]


# ---------------------------------------------------------------------------
# 1. textbook layer from torch library routines + autograd (independent path)
# ---------------------------------------------------------------------------
def torch_rope(x, base):
    """Rotation written with complex numbers: (x1 + i x2) * exp(i p theta)."""
    s, n, d = x.shape
    half = d // 2
    theta = base ** (-torch.arange(half, dtype=torch.float64) * 2.0 / d)
    ang = torch.arange(s, dtype=torch.float64)[:, None] * theta[None, :]
    z = torch.complex(x[..., :half], x[..., half:]) * torch.polar(torch.ones_like(ang), ang)[:, None, :]
    return torch.cat([z.real, z.imag], dim=-1)


def torch_layer(cfg, W, X):
    """Ordinary unsharded pre-norm layer: X + Attn(N(X)), then + MLP(N(.))."""
    h, n, d = cfg.hidden, cfg.heads_local, cfg.head_dim
    a = n * d
    s = X.shape[0]

    def norm(x, g, b):
        if cfg.norm == "ln":
            return F.layer_norm(x, (h,), g, b, cfg.eps)
        return F.rms_norm(x, (h,), g, cfg.eps)

    xl = norm(X, W["norm1_g"], W.get("norm1_b"))
    qkv = xl @ W["w_qkv"] + (W["b_qkv"] if cfg.has_bias else 0)
    nk = cfg.kv_heads
    q = qkv[:, :a].reshape(s, n, d)
    k, v = (qkv[:, a + i * nk * d:a + (i + 1) * nk * d].reshape(s, nk, d) for i in range(2))
    if cfg.rope:
        q, k = torch_rope(q, cfg.rope_base), torch_rope(k, cfg.rope_base)
    # grouped-query attention written as ordinary attention over key / value heads repeated per group
    k, v = k.repeat_interleave(n // nk, dim=1), v.repeat_interleave(n // nk, dim=1)
    ctx = F.scaled_dot_product_attention(q.transpose(0, 1)[None], k.transpose(0, 1)[None],
                                         v.transpose(0, 1)[None], is_causal=cfg.causal)[0]
    ctx = ctx.transpose(0, 1).reshape(s, a)
    xa = X + ctx @ W["w_o"] + (W["b_o"] if cfg.has_bias else 0)
    zl = norm(xa, W["norm2_g"], W.get("norm2_b"))
    h1 = zl @ W["w_fc1"] + (W["b_fc1"] if cfg.has_bias else 0)
    g = F.gelu(h1) if cfg.act == "gelu" else F.silu(h1) * (zl @ W["w_up"])
    return xa + g @ W["w_fc2"] + (W["b_fc2"] if cfg.has_bias else 0)


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("t,heads,kv", [(1, 4, 0), (2, 4, 0), (4, 4, 0), (1, 6, 2), (2, 8, 2), (2, 8, 4), (4, 12, 4)])
def test_tp_sum_equals_textbook_layer_and_autograd(variant, t, heads, kv):
    """Eq. 1-2: summing the t rank partials at the AR points reproduces the unsharded
    layer and its gradients; shard weight grads are slices of the unsharded ones.
    kv > 0: grouped-query attention (heads / kv query heads share a key / value head)."""
    rng = np.random.default_rng(7)
    cfg = O.LayerCfg(hidden=24, heads_local=heads, head_dim=8, ffn_local=32, tp=1, kv_heads_local=kv, **variant)
    s = 11
    W = rand_weights(cfg, rng)
    X = rng.standard_normal((s, cfg.hidden))
    R = rng.standard_normal((s, cfg.hidden))

    Wt = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in W.items()}
    Xt = torch.tensor(X, dtype=torch.float64, requires_grad=True)
    out_t = torch_layer(cfg, Wt, Xt)
    (out_t * torch.tensor(R)).sum().backward()

    shards = [O.shard_weights(cfg, W, t, r) for r in range(t)]
    cfg_r = shards[0][0]
    ws = [w for _, w in shards]
    out, stashes = O.layer_forward_all_ranks(cfg_r, ws, X)
    np.testing.assert_allclose(out, out_t.detach().numpy(), rtol=1e-10, atol=1e-10)
    dX, grads = O.layer_backward_all_ranks(cfg_r, ws, stashes, R)
    np.testing.assert_allclose(dX, Xt.grad.numpy(), rtol=1e-9, atol=1e-10)

    a, f, ak = cfg.attn_local, cfg.ffn_local, cfg.kv_local
    al, fl, akl = a // t, f // t, ak // t
    for r in range(t):
        g = grads[r]
        full = {k: v.grad.numpy() for k, v in Wt.items()}
        cols = np.concatenate([np.arange(r * al, (r + 1) * al), np.arange(a + r * akl, a + (r + 1) * akl),
                               np.arange(a + ak + r * akl, a + ak + (r + 1) * akl)])
        np.testing.assert_allclose(g["w_qkv"], full["w_qkv"][:, cols], rtol=1e-9, atol=1e-10)
        np.testing.assert_allclose(g["w_o"], full["w_o"][r * al:(r + 1) * al], rtol=1e-9, atol=1e-10)
        np.testing.assert_allclose(g["w_fc1"], full["w_fc1"][:, r * fl:(r + 1) * fl], rtol=1e-9, atol=1e-10)
        np.testing.assert_allclose(g["w_fc2"], full["w_fc2"][r * fl:(r + 1) * fl], rtol=1e-9, atol=1e-10)
        if cfg.act == "swiglu":
            np.testing.assert_allclose(g["w_up"], full["w_up"][:, r * fl:(r + 1) * fl], rtol=1e-9, atol=1e-10)
        for key in ("norm1_g", "norm2_g") + (("norm1_b", "norm2_b") if cfg.norm == "ln" else ()):
            np.testing.assert_allclose(g[key], full[key], rtol=1e-9, atol=1e-10)
        if cfg.has_bias:
            np.testing.assert_allclose(g["b_qkv"], full["b_qkv"][cols], rtol=1e-9, atol=1e-10)
            np.testing.assert_allclose(g["b_fc1"], full["b_fc1"][r * fl:(r + 1) * fl], rtol=1e-9, atol=1e-10)
    if cfg.has_bias:  # replicated biases carry 1/t each: their rank-sum is the full gradient
        for key in ("b_o", "b_fc2"):
            np.testing.assert_allclose(sum(g[key] for g in grads), Wt[key].grad.numpy(),
                                       rtol=1e-9, atol=1e-10)


# ---------------------------------------------------------------------------
# 2. central finite differences of the all-rank layer
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("variant", VARIANTS[:3])
@pytest.mark.parametrize("t", [1, 2])
def test_finite_differences(variant, t):
    rng = np.random.default_rng(3)
    cfg = O.LayerCfg(hidden=8, heads_local=2, head_dim=4, ffn_local=16, tp=1, **variant)
    s = 5
    W = rand_weights(cfg, rng)
    X = rng.standard_normal((s, cfg.hidden))
    R = rng.standard_normal((s, cfg.hidden))

    def loss(Wd, Xd):
        sh = [O.shard_weights(cfg, Wd, t, r) for r in range(t)]
        out, _ = O.layer_forward_all_ranks(sh[0][0], [w for _, w in sh], Xd)
        return float((out * R).sum())

    sh = [O.shard_weights(cfg, W, t, r) for r in range(t)]
    out, st = O.layer_forward_all_ranks(sh[0][0], [w for _, w in sh], X)
    dX, grads = O.layer_backward_all_ranks(sh[0][0], [w for _, w in sh], st, R)

    eps = 1e-6
    for idx in [(0, 0), (2, 3), (4, 7), (1, 5)]:
        Xp, Xm = X.copy(), X.copy()
        Xp[idx] += eps
        Xm[idx] -= eps
        fd = (loss(W, Xp) - loss(W, Xm)) / (2 * eps)
        assert abs(fd - dX[idx]) < 1e-6 * max(1.0, abs(fd))

    # weight gradients of rank 0 against finite differences on the unsharded tensors
    cfg_r = sh[0][0]
    al, fl, a = cfg_r.attn_local, cfg_r.ffn_local, cfg.attn_local
    probes = [("w_qkv", (3, 1), (3, 1)), ("w_qkv", (5, al + 1), (5, a + 1)),
              ("w_qkv", (2, 2 * al), (2, 2 * a)), ("w_o", (1, 4), (1, 4)),
              ("w_fc1", (6, 2), (6, 2)), ("w_fc2", (3, 5), (3, 5)),
              ("norm1_g", (4,), (4,)), ("norm2_g", (1,), (1,))]
    if cfg.norm == "ln":
        probes += [("norm1_b", (2,), (2,)), ("norm2_b", (7,), (7,))]
    if cfg.act == "swiglu":
        probes.append(("w_up", (0, 3), (0, 3)))
    if cfg.has_bias:
        probes += [("b_qkv", (al + 2,), (a + 2,)), ("b_fc1", (1,), (1,))]
    for key, loc, full in probes:
        Wp = {k: v.copy() for k, v in W.items()}
        Wm = {k: v.copy() for k, v in W.items()}
        Wp[key][full] += eps
        Wm[key][full] -= eps
        fd = (loss(Wp, X) - loss(Wm, X)) / (2 * eps)
        assert abs(fd - grads[0][key][loc]) < 2e-6 * max(1.0, abs(fd)), (key, fd, grads[0][key][loc])
    if cfg.has_bias:
        for key in ("b_o", "b_fc2"):
            Wp = {k: v.copy() for k, v in W.items()}
            Wm = {k: v.copy() for k, v in W.items()}
            Wp[key][3] += eps
            Wm[key][3] -= eps
            fd = (loss(Wp, X) - loss(Wm, X)) / (2 * eps)
            assert abs(fd - sum(g[key][3] for g in grads)) < 2e-6 * max(1.0, abs(fd))


def test_finite_differences_grouped_query():
    """Central differences of a 2-rank layer with 4 query heads over 2 key / value heads: dX and the gradient
    of the K and V columns of the QKV weight (which collect the contributions of a whole head group)."""
    rng = np.random.default_rng(4)
    cfg = O.LayerCfg(hidden=8, heads_local=4, head_dim=4, ffn_local=16, tp=1, kv_heads_local=2, rope=True)
    s, t = 5, 2
    W = rand_weights(cfg, rng)
    X = rng.standard_normal((s, cfg.hidden))
    R = rng.standard_normal((s, cfg.hidden))

    def loss(Wd, Xd):
        sh = [O.shard_weights(cfg, Wd, t, r) for r in range(t)]
        out, _ = O.layer_forward_all_ranks(sh[0][0], [w for _, w in sh], Xd)
        return float((out * R).sum())

    sh = [O.shard_weights(cfg, W, t, r) for r in range(t)]
    out, st = O.layer_forward_all_ranks(sh[0][0], [w for _, w in sh], X)
    dX, grads = O.layer_backward_all_ranks(sh[0][0], [w for _, w in sh], st, R)
    eps = 1e-6
    for idx in [(0, 0), (3, 5), (4, 2)]:
        Xp, Xm = X.copy(), X.copy()
        Xp[idx] += eps
        Xm[idx] -= eps
        fd = (loss(W, Xp) - loss(W, Xm)) / (2 * eps)
        assert abs(fd - dX[idx]) < 1e-6 * max(1.0, abs(fd))
    a, ak = cfg.attn_local, cfg.kv_local          # 16, 8: rank 0 holds Q cols 0..7, K cols 16..19, V cols 24..27
    al, akl = a // t, ak // t
    for loc, full in [((2, 1), (2, 1)), ((5, al + 2), (5, a + 2)), ((1, al + akl + 3), (1, a + ak + 3))]:
        Wp = {k: v.copy() for k, v in W.items()}
        Wm = {k: v.copy() for k, v in W.items()}
        Wp["w_qkv"][full] += eps
        Wm["w_qkv"][full] -= eps
        fd = (loss(Wp, X) - loss(Wm, X)) / (2 * eps)
        assert abs(fd - grads[0]["w_qkv"][loc]) < 2e-6 * max(1.0, abs(fd)), (loc, fd, grads[0]["w_qkv"][loc])


# ---------------------------------------------------------------------------
# 3. B units + W units == independently written fused backward
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("t,heads,kv", [(1, 2, 0), (2, 2, 0), (8, 2, 0), (4, 6, 2), (8, 5, 1)])
def test_b_plus_w_equals_fused_backward(variant, t, heads, kv):
    """Single rank, identity at the AR points (the configuration the GPU is timed in)."""
    rng = np.random.default_rng(11)
    cfg = O.LayerCfg(hidden=16, heads_local=heads, head_dim=8, ffn_local=24, tp=t, kv_heads_local=kv, **variant)
    s = 9
    W = rand_weights(cfg, rng)
    X = rng.standard_normal((s, cfg.hidden))
    dO = rng.standard_normal((s, cfg.hidden))
    st = {}
    O.forward_unit(cfg, O.PRE_ATTN, W, st, x_in=X)
    xa = O.forward_unit(cfg, O.ATTN, W, st, x_resid=X)
    O.forward_unit(cfg, O.PRE_MLP, W, st, x_in=xa)
    O.forward_unit(cfg, O.MLP, W, st, x_resid=xa)
    g = {}
    dz = O.backward_input_unit(cfg, O.MLP, W, st, dO)
    dxa = O.backward_input_unit(cfg, O.PRE_MLP, W, st, dz, d_resid=dO, grads=g)
    dxl = O.backward_input_unit(cfg, O.ATTN, W, st, dxa)
    dx = O.backward_input_unit(cfg, O.PRE_ATTN, W, st, dxl, d_resid=dxa, grads=g)
    O.backward_weight_unit(cfg, O.ATTN, st, dxa, g)
    O.backward_weight_unit(cfg, O.MLP, st, dO, g)
    dx_f, g_f = O.fused_layer_backward(cfg, W, X, dO)
    np.testing.assert_allclose(dx, dx_f, rtol=1e-12, atol=1e-12)
    assert set(g) == set(g_f)
    for key in g:
        np.testing.assert_allclose(g[key], g_f[key], rtol=1e-12, atol=1e-12, err_msg=key)


def test_weight_grads_accumulate_over_microbatches():
    rng = np.random.default_rng(5)
    cfg = O.LayerCfg(hidden=8, heads_local=2, head_dim=4, ffn_local=12, tp=1)
    W = rand_weights(cfg, rng)
    acc, singles = {}, []
    for mb in range(3):
        X, dO = rng.standard_normal((6, 8)), rng.standard_normal((6, 8))
        out, st = O.layer_forward_all_ranks(cfg, [W], X)
        _, g1 = O.layer_backward_all_ranks(cfg, [W], st, dO)
        singles.append(g1[0])
        dxa = O.backward_input_unit(cfg, O.PRE_MLP, W, st[0], st[0]["dh"] @ W["w_fc1"].T, d_resid=dO)
        O.backward_weight_unit(cfg, O.MLP, st[0], dO, acc)
        O.backward_weight_unit(cfg, O.ATTN, st[0], dxa, acc)
    for key in acc:
        np.testing.assert_allclose(acc[key], sum(s_[key] for s_ in singles), rtol=1e-12, atol=1e-12)


# ---------------------------------------------------------------------------
# 4. brute force with scalar loops, closed forms, special cases
# ---------------------------------------------------------------------------
def test_attention_brute_force_loops():
    rng = np.random.default_rng(0)
    s, n, d = 6, 2, 4
    q, k, v = (rng.standard_normal((s, n, d)) for _ in range(3))
    for causal in (True, False):
        got = O.attention_fwd(q, k, v, causal)
        for hd in range(n):
            for i in range(s):
                js = range(i + 1) if causal else range(s)
                sc = [sum(q[i, hd, c] * k[j, hd, c] for c in range(d)) / math.sqrt(d) for j in js]
                m = max(sc)
                e = [math.exp(x - m) for x in sc]
                z = sum(e)
                for c in range(d):
                    want = sum(e[jj] / z * v[j, hd, c] for jj, j in enumerate(js))
                    assert abs(got[i, hd, c] - want) < 1e-12


def test_grouped_query_attention_is_attention_over_repeated_heads():
    """n query heads over n_kv key / value heads equals ordinary attention with every key / value head repeated
    n / n_kv times; the gradient of a shared head is the sum over its group.  (The multi-head path used on the
    right-hand side is pinned by the brute-force and library tests.)"""
    rng = np.random.default_rng(21)
    s, n, nk, d = 9, 6, 2, 4
    q, dctx = rng.standard_normal((s, n, d)), rng.standard_normal((s, n, d))
    k, v = rng.standard_normal((s, nk, d)), rng.standard_normal((s, nk, d))
    kr, vr = np.repeat(k, n // nk, axis=1), np.repeat(v, n // nk, axis=1)
    for causal in (True, False):
        np.testing.assert_allclose(O.attention_fwd(q, k, v, causal), O.attention_fwd(q, kr, vr, causal), rtol=1e-12)
        dq, dk, dv = O.attention_bwd(q, k, v, dctx, causal)
        dq_r, dk_r, dv_r = O.attention_bwd(q, kr, vr, dctx, causal)
        np.testing.assert_allclose(dq, dq_r, rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(dk, dk_r.reshape(s, nk, n // nk, d).sum(axis=2), rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(dv, dv_r.reshape(s, nk, n // nk, d).sum(axis=2), rtol=1e-12, atol=1e-13)
    # a wrong head-to-group map (i % n_kv instead of i // group) changes the result
    assert not np.allclose(O.attention_fwd(q, k, v, True), O.attention_fwd(q, np.tile(k, (1, n // nk, 1)), np.tile(v, (1, n // nk, 1)), True))


def test_attention_special_cases():
    rng = np.random.default_rng(1)
    q, k, v = (rng.standard_normal((7, 3, 8)) for _ in range(3))
    ctx = O.attention_fwd(q, k, v, True)
    np.testing.assert_allclose(ctx[0], v[0], atol=1e-14)             # causal row 0 sees only key 0
    one = O.attention_fwd(q[:1], k[:1], v[:1], False)
    np.testing.assert_allclose(one, v[:1], atol=1e-14)               # s = 1
    P = O._probs(q[:, 0], k[:, 0], True)
    np.testing.assert_allclose(P.sum(1), 1.0, atol=1e-14)
    assert np.all(np.triu(P, 1) == 0)
    # uniform keys -> bidirectional context is the mean of the values
    ku = np.repeat(k[:1], 7, axis=0)
    np.testing.assert_allclose(O.attention_fwd(q, ku, v, False),
                               np.broadcast_to(v.mean(0), v.shape), atol=1e-13)
    # dS rows sum to zero => shifting all keys by a constant vector leaves dq unchanged,
    # and sum_j dS_ij = 0 makes dk sum to zero when all queries are equal
    dctx = rng.standard_normal(q.shape)
    qe = np.repeat(q[:1], 7, axis=0)
    _, dk, _ = O.attention_bwd(qe, k, v, dctx, False)
    np.testing.assert_allclose(dk.sum(0), 0.0, atol=1e-12)


def test_norm_closed_forms_and_library():
    rng = np.random.default_rng(2)
    X = rng.standard_normal((5, 16)) * 3 + 1
    ln = O.LayerCfg(8, 1, 8, 8, norm="ln")
    Y = O.norm_fwd(ln, X, np.ones(16), np.zeros(16))
    np.testing.assert_allclose(Y.mean(1), 0, atol=1e-14)
    v = X.var(1)
    np.testing.assert_allclose(Y.var(1), v / (v + ln.eps), rtol=1e-12)
    g, b = rng.standard_normal(16), rng.standard_normal(16)
    want = F.layer_norm(torch.tensor(X), (16,), torch.tensor(g), torch.tensor(b), ln.eps).numpy()
    np.testing.assert_allclose(O.norm_fwd(ln, X, g, b), want, rtol=1e-12, atol=1e-12)
    dX, _, db = O.norm_bwd(ln, rng.standard_normal((5, 16)), X, g)
    np.testing.assert_allclose(dX.sum(1), 0, atol=1e-13)             # LN output is shift invariant
    rms = replace(ln, norm="rms")
    # scaling the input by c>0 leaves RMSNorm (eps -> 0) unchanged; loop definition
    rms0 = replace(rms, eps=0.0)
    np.testing.assert_allclose(O.norm_fwd(rms0, 4.0 * X, g), O.norm_fwd(rms0, X, g), rtol=1e-13)
    for i in range(5):
        r = math.sqrt(sum(x * x for x in X[i]) / 16 + rms.eps)
        np.testing.assert_allclose(O.norm_fwd(rms, X, g)[i], X[i] / r * g, rtol=1e-13)


def test_gelu_against_printed_normal_cdf_table():
    rows = [ln.split() for ln in open(os.path.join(HERE, "golden", "normal_cdf.txt"))
            if ln.strip() and not ln.startswith("#")]
    for xs, ps in rows:
        x, p = float(xs), float(ps)
        assert abs(O.gelu(np.array(x)) - x * p) < 1e-9 * max(1, abs(x))
        phi = math.exp(-x * x / 2) / math.sqrt(2 * math.pi)
        assert abs(O.gelu_grad(np.array(x)) - (p + x * phi)) < 1e-9
    assert O.gelu(np.array(0.0)) == 0.0 and O.gelu_grad(np.array(0.0)) == 0.5
    x = np.linspace(-4, 4, 33)
    np.testing.assert_allclose(O.gelu(x), [0.5 * v * (1 + math.erf(v / math.sqrt(2))) for v in x], rtol=1e-13)
    np.testing.assert_allclose(O.silu(x), F.silu(torch.tensor(x)).numpy(), rtol=1e-13)
    e = 1e-6
    np.testing.assert_allclose(O.silu_grad(x), (O.silu(x + e) - O.silu(x - e)) / (2 * e), atol=1e-8)
    np.testing.assert_allclose(O.gelu_grad(x), (O.gelu(x + e) - O.gelu(x - e)) / (2 * e), atol=1e-8)


def test_rope_properties():
    rng = np.random.default_rng(4)
    s, n, d = 9, 2, 8
    x, y = rng.standard_normal((s, n, d)), rng.standard_normal((s, n, d))
    rx = O.rope(x, 10000.0)
    np.testing.assert_allclose(rx[0], x[0], atol=1e-15)                       # position 0: identity
    half = d // 2
    np.testing.assert_allclose(rx[..., :half] ** 2 + rx[..., half:] ** 2,
                               x[..., :half] ** 2 + x[..., half:] ** 2, rtol=1e-12)
    np.testing.assert_allclose(O.rope(rx, 10000.0, inverse=True), x, atol=1e-13)
    # <R_m q, R_n k> depends only on m-n: place the same q,k at two position pairs
    q0, k0 = rng.standard_normal(d), rng.standard_normal(d)
    Q = np.tile(q0, (s, 1, 1))
    K = np.tile(k0, (s, 1, 1))
    rq, rk = O.rope(Q, 10000.0), O.rope(K, 10000.0)
    assert abs(rq[5, 0] @ rk[2, 0] - rq[8, 0] @ rk[5, 0]) < 1e-12
    # explicit scalar formula for one element: pair (1, 1+half) of token 3
    th = 3 * 10000.0 ** (-2.0 * 1 / d)
    assert abs(rx[3, 1, 1] - (x[3, 1, 1] * math.cos(th) - x[3, 1, 1 + half] * math.sin(th))) < 1e-13
    assert abs(rx[3, 1, 1 + half] - (x[3, 1, 1 + half] * math.cos(th) + x[3, 1, 1] * math.sin(th))) < 1e-13
    np.testing.assert_allclose(rx, torch_rope(torch.tensor(x), 10000.0).numpy(), atol=1e-13)


@pytest.mark.parametrize("t", [1, 4])
def test_zero_weights_leave_pure_residual(t):
    """With all linear weights zero a unit returns X/t and passes dX_attn straight (Eq. 1-2)."""
    rng = np.random.default_rng(9)
    cfg = O.LayerCfg(hidden=8, heads_local=2, head_dim=4, ffn_local=8, tp=t, has_bias=False)
    W = {k: np.zeros_like(v) if k.startswith("w_") else v for k, v in rand_weights(cfg, rng).items()}
    X = rng.standard_normal((4, 8))
    st = {}
    O.forward_unit(cfg, O.PRE_ATTN, W, st, x_in=X)
    y = O.forward_unit(cfg, O.ATTN, W, st, x_resid=X)
    np.testing.assert_allclose(y, X / t, atol=1e-15)
    O.forward_unit(cfg, O.PRE_MLP, W, st, x_in=X)
    np.testing.assert_allclose(O.forward_unit(cfg, O.MLP, W, st, x_resid=X), X / t, atol=1e-15)
    dxa = rng.standard_normal((4, 8))
    dxl = O.backward_input_unit(cfg, O.ATTN, W, st, dxa)
    np.testing.assert_allclose(dxl, 0, atol=1e-15)
    dx = O.backward_input_unit(cfg, O.PRE_ATTN, W, st, dxl, d_resid=dxa)
    np.testing.assert_allclose(dx, dxa, atol=1e-15)


# ---- the stand-alone row softmax ------------------------------------------------------------------------------
def test_softmax_against_torch_and_its_closed_forms():
    rng = np.random.default_rng(11)
    x = rng.standard_normal((12, 6)) * 3
    dy = rng.standard_normal((12, 6))
    for scale in (1.0, 0.35):
        xt = torch.tensor(x, dtype=torch.float64, requires_grad=True)
        yt = torch.softmax(xt * scale, dim=1)
        yt.backward(torch.tensor(dy))
        y = O.softmax_fwd(x, scale)
        np.testing.assert_allclose(y, yt.detach().numpy(), rtol=1e-13, atol=1e-15)
        np.testing.assert_allclose(O.softmax_bwd(y, dy, scale), xt.grad.numpy(), rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(y.sum(1), 1.0, rtol=1e-14)                      # rows are distributions
        np.testing.assert_allclose(O.softmax_bwd(y, dy, scale).sum(1), 0.0, atol=1e-14)   # shifts of a row change nothing
    # a constant row is uniform; adding a constant to a row changes nothing; a far larger entry takes everything
    np.testing.assert_allclose(O.softmax_fwd(np.full((2, 5), 7.0)), 0.2, rtol=1e-15)
    np.testing.assert_allclose(O.softmax_fwd(x + 100.0), O.softmax_fwd(x), rtol=1e-12)
    big = np.zeros((1, 4)); big[0, 2] = 800.0
    np.testing.assert_allclose(O.softmax_fwd(big), [[0, 0, 1, 0]], atol=1e-300)
    # central differences of sum(y * R)
    R = rng.standard_normal(x.shape)
    g = O.softmax_bwd(O.softmax_fwd(x, 0.7), R, 0.7)
    for (i, j) in [(0, 0), (5, 3), (11, 5)]:
        h = 1e-6
        xp, xm = x.copy(), x.copy()
        xp[i, j] += h; xm[i, j] -= h
        fd = ((O.softmax_fwd(xp, 0.7) * R).sum() - (O.softmax_fwd(xm, 0.7) * R).sum()) / (2 * h)
        assert abs(fd - g[i, j]) < 1e-8


def test_causal_softmax_masks_keys_after_the_query():
    rng = np.random.default_rng(12)
    n = 5
    x = rng.standard_normal((2 * n, n))          # two stacked [n, n] squares
    y = O.softmax_fwd(x, 0.5, causal=True)
    for r in range(2 * n):
        i = r % n
        assert np.all(y[r, i + 1:] == 0.0)
        e = np.exp(0.5 * (x[r, :i + 1] - x[r, :i + 1].max()))      # the unmasked prefix, by its own definition
        np.testing.assert_allclose(y[r, :i + 1], e / e.sum(), rtol=1e-14)
    np.testing.assert_allclose(y[0], [1, 0, 0, 0, 0], atol=0)       # the first query sees only its own key
    # and it is the normalisation the attention oracle applies to q k^T / sqrt(d)
    q, k = rng.standard_normal((n, 8)), rng.standard_normal((n, 8))
    np.testing.assert_allclose(O.softmax_fwd(q @ k.T, 1 / np.sqrt(8), causal=True), O._probs(q, k, True), rtol=1e-13)

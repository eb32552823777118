"""Pins for the CPU oracle: it is checked against things other than itself.

The paper prints no worked numerical example of the layer, so the pins are
(1) central finite differences of the scalar L = sum(Y * dY), (2) invariants,
(3) structural properties, (4) special cases with closed forms, (5) PyTorch's
CPU float64 encoder layer with autograd, (6) a loop-only scalar implementation
on a tiny shape.  A dropped term, a wrong sign, a transposed operand or a wrong
index in oracle/oracle.py fails at least one of them.
"""
import math

import numpy as np
import pytest

from oracle import oracle as orc
from workloads import CONFIGS, PARAM_NAMES, make_inputs

CFG1 = CONFIGS["cfg1_tiny_f32"]


def _inputs(cfg, seed=0, lengths=None):
    inp = make_inputs(cfg, seed=seed, nontrivial=True)
    if lengths is not None:
        inp["lengths"] = np.asarray(lengths, np.int32)
    return inp


def _loss(p, X, dY, lengths, kw):
    Y, _ = orc.layer_forward(p, X, lengths, **kw)
    return float(np.sum(Y * dY))


# ---------------------------------------------------------------- (1) finite differences
@pytest.mark.parametrize("norm", ["post", "pre"])
@pytest.mark.parametrize("act", ["relu", "gelu"])
@pytest.mark.parametrize("masked", [False, True])
def test_finite_differences(norm, act, masked):
    cfg = CFG1
    lengths = [11, 5] if masked else None
    inp = _inputs(cfg, seed=3, lengths=lengths)
    kw = dict(heads=cfg.H, act=act, norm=norm, eps=cfg.eps)
    p = {k: v.astype(np.float64) for k, v in inp["params"].items()}
    X, dY = inp["X"].astype(np.float64), inp["dY"].astype(np.float64)
    L = inp["lengths"]
    Y, dX, g = orc.layer_forward_backward(p, X, dY, L, **kw)
    _, cache = orc.layer_forward(p, X, L, **kw)
    U = cache["ffn"]["U"]
    assert np.min(np.abs(U)) > 1e-5 or act == "gelu", "a pre-activation sits on the ReLU kink"
    rng = np.random.default_rng(11)
    h = 1e-6

    def check(name, arr, grad, n):
        flat = arr.reshape(-1)
        idx = rng.choice(flat.size, size=min(n, flat.size), replace=False)
        scale = np.max(np.abs(grad)) + 1e-30
        for i in idx:
            old = flat[i]
            flat[i] = old + h
            lp = _loss(p, X, dY, L, kw)
            flat[i] = old - h
            lm = _loss(p, X, dY, L, kw)
            flat[i] = old
            fd = (lp - lm) / (2 * h)
            assert abs(fd - grad.reshape(-1)[i]) <= 2e-6 * scale, (name, int(i), fd, grad.reshape(-1)[i])

    check("X", X, dX, 60)
    for name in PARAM_NAMES:
        check(name, p[name], g[name], 25)


# ---------------------------------------------------------------- (2) invariants
def test_softmax_rows_and_mask():
    cfg = CFG1
    inp = _inputs(cfg, lengths=[9, 16])
    Y, c = orc.layer_forward(inp["params"], inp["X"], inp["lengths"], heads=cfg.H)
    P = c["attn"]["P"]
    assert np.allclose(P.sum(-1), 1.0, atol=1e-14)
    assert np.all(P[0, :, :, 9:] == 0.0)
    assert np.all(P[1] > 0.0)
    assert np.all(P >= 0.0)


def test_layernorm_statistics():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((7, 64)) * 3 + 2
    eps = 1e-5
    y, xhat, rstd = orc.layernorm_fwd(x, np.ones(64), np.zeros(64), eps)
    assert np.allclose(y.mean(-1), 0, atol=1e-14)
    var = x.var(-1)
    assert np.allclose(y.var(-1), var / (var + eps), rtol=1e-12)
    # textbook value on one row computed with the statistics module's definitions
    r = x[3]
    mu = sum(r) / 64
    v = sum((t - mu) ** 2 for t in r) / 64
    assert np.allclose(y[3], [(t - mu) / math.sqrt(v + eps) for t in r], atol=1e-13)


def test_gradient_orthogonality():
    cfg = CFG1
    inp = _inputs(cfg)
    rng = np.random.default_rng(5)
    dy = rng.standard_normal((4, 9, 64))
    x = rng.standard_normal((4, 9, 64))
    g = 1 + 0.1 * rng.standard_normal(64)
    _, xhat, rstd = orc.layernorm_fwd(x, g, np.zeros(64), 1e-5)
    dx, dg, db = orc.layernorm_bwd(dy, xhat, rstd, g)
    assert np.allclose(dx.sum(-1), 0, atol=1e-12)
    # sum_j dx_j xhat_j = rstd * sum(g xhat) * eps / (var + eps): zero only in the limit eps -> 0
    var = x.var(-1)
    want = rstd[..., 0] * (dy * g * xhat).sum(-1) * 1e-5 / (var + 1e-5)
    assert np.allclose((dx * xhat).sum(-1), want, atol=1e-12)
    # rows of dS sum to zero: dQ is orthogonal to nothing in general, so test dS via a K of ones
    B, H, T, dh = 2, 2, 5, 4
    Q, K, V, dO = (rng.standard_normal((B, H, T, dh)) for _ in range(4))
    O, P = orc.attention_fwd(Q, K, V, [3, 5])
    dQ, dK, dV = orc.attention_bwd(dO, Q, np.ones_like(K), V, P)
    assert np.allclose(dQ, 0, atol=1e-13)          # dQ = rowsum(dS) * 1 / sqrt(dh)
    dQ, dK, dV = orc.attention_bwd(dO, Q, K, V, P)
    assert np.all(dK[0, :, 3:] == 0) and np.all(dV[0, :, 3:] == 0)
    assert np.any(dK[1, :, 3:] != 0)


# ---------------------------------------------------------------- (3) structure
@pytest.mark.parametrize("norm", ["post", "pre"])
def test_permutation_equivariance_and_batch_independence(norm):
    cfg = CFG1
    inp = _inputs(cfg, seed=1)
    kw = dict(heads=cfg.H, act="gelu", norm=norm)
    X, dY, p = inp["X"], inp["dY"], inp["params"]
    Y, dX, g = orc.layer_forward_backward(p, X, dY, None, **kw)
    perm = np.random.default_rng(2).permutation(cfg.T)
    Yp, dXp, gp = orc.layer_forward_backward(p, X[:, perm], dY[:, perm], None, **kw)
    assert np.allclose(Yp, Y[:, perm], atol=1e-12)
    assert np.allclose(dXp, dX[:, perm], atol=1e-12)
    for k in PARAM_NAMES:
        assert np.allclose(gp[k], g[k], atol=1e-11)
    X2 = X.copy()
    X2[1] += 1.0
    Y2, _ = orc.layer_forward(p, X2, None, **kw)
    assert np.array_equal(Y2[0], Y[0]) and not np.allclose(Y2[1], Y[1])


def test_padded_keys_do_not_influence_other_rows():
    cfg = CFG1
    inp = _inputs(cfg, lengths=[7, 16])
    kw = dict(heads=cfg.H, act="relu", norm="post")
    X, p, L = inp["X"].astype(np.float64), inp["params"], inp["lengths"]
    Y, _ = orc.layer_forward(p, X, L, **kw)
    X2 = X.copy()
    X2[0, 10] += 5.0                       # a padded position of sequence 0
    Y2, _ = orc.layer_forward(p, X2, L, **kw)
    rows = [i for i in range(cfg.T) if i != 10]
    assert np.array_equal(Y2[0, rows], Y[0, rows])
    assert not np.allclose(Y2[0, 10], Y[0, 10])
    X3 = X.copy()
    X3[0, 3] += 5.0                        # a valid key: every row of sequence 0 moves
    Y3, _ = orc.layer_forward(p, X3, L, **kw)
    assert np.all(np.abs(Y3[0] - Y[0]).max(-1) > 0)


def test_lengths_none_equals_full_lengths():
    cfg = CFG1
    inp = _inputs(cfg)
    kw = dict(heads=cfg.H, act="relu", norm="post")
    a = orc.layer_forward_backward(inp["params"], inp["X"], inp["dY"], None, **kw)
    b = orc.layer_forward_backward(inp["params"], inp["X"], inp["dY"], [cfg.T] * cfg.B, **kw)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    with pytest.raises(ValueError):
        orc.layer_forward(inp["params"], inp["X"], [0, 3], **kw)


# ---------------------------------------------------------------- (4) closed forms
def test_uniform_attention_when_wq_is_zero():
    cfg = CFG1
    inp = _inputs(cfg, lengths=[6, 16])
    p = {k: v.astype(np.float64).copy() for k, v in inp["params"].items()}
    D = cfg.D
    p["Wqkv"][:D] = 0
    p["bqkv"][:D] = 0
    X = inp["X"].astype(np.float64)
    _, c = orc.layer_forward(p, X, inp["lengths"], heads=cfg.H)
    V = X @ p["Wqkv"][2 * D:].T + p["bqkv"][2 * D:]
    want0 = V[0, :6].mean(0)
    want1 = V[1].mean(0)
    assert np.allclose(c["attn"]["O"][0], want0[None, :], atol=1e-13)
    assert np.allclose(c["attn"]["O"][1], want1[None, :], atol=1e-13)


def test_single_token_sequence_is_affine_chain():
    cfg = CFG1.with_(T=1)
    inp = make_inputs(cfg, seed=4, nontrivial=True)
    p = {k: v.astype(np.float64) for k, v in inp["params"].items()}
    X = inp["X"].astype(np.float64)
    D = cfg.D
    Y, _ = orc.layer_forward(p, X, None, heads=cfg.H, act="relu", norm="pre", eps=1e-5)

    def ln(r, g, b):
        mu = r.mean(-1, keepdims=True)
        return g * (r - mu) / np.sqrt(((r - mu) ** 2).mean(-1, keepdims=True) + 1e-5) + b
    n1 = ln(X, p["ln1_g"], p["ln1_b"])
    v = n1 @ p["Wqkv"][2 * D:].T + p["bqkv"][2 * D:]          # P == 1  =>  O == V
    r1 = X + v @ p["Wo"].T + p["bo"]
    n2 = ln(r1, p["ln2_g"], p["ln2_b"])
    want = r1 + np.maximum(n2 @ p["W1"].T + p["b1"], 0) @ p["W2"].T + p["b2"]
    assert np.allclose(Y, want, atol=1e-12)


def test_zeroed_branches():
    cfg = CFG1
    inp = _inputs(cfg)
    X = inp["X"].astype(np.float64)
    p = {k: v.astype(np.float64).copy() for k, v in inp["params"].items()}
    p["W2"][:] = 0
    p["b2"][:] = 0
    p["Wo"][:] = 0
    p["bo"][:] = 0
    Ypre, _ = orc.layer_forward(p, X, None, heads=cfg.H, norm="pre")
    assert np.array_equal(Ypre, X)
    Ypost, _ = orc.layer_forward(p, X, None, heads=cfg.H, norm="post")
    y1, _, _ = orc.layernorm_fwd(X, p["ln1_g"], p["ln1_b"], 1e-5)
    y2, _, _ = orc.layernorm_fwd(y1, p["ln2_g"], p["ln2_b"], 1e-5)
    assert np.allclose(Ypost, y2, atol=1e-13)


def test_gelu_values_and_derivative():
    # Phi(1) = 0.841344746068543 (standard normal table), phi(1) = 0.24197072451914337
    assert abs(orc.gelu_fwd(np.array([1.0]))[0] - 0.841344746068543) < 1e-15
    assert abs(orc.gelu_bwd(np.array([1.0]), np.array([1.0]))[0] - (0.841344746068543 + 0.24197072451914337)) < 1e-15
    assert orc.gelu_fwd(np.array([0.0]))[0] == 0.0
    assert abs(orc.gelu_bwd(np.array([1.0]), np.array([0.0]))[0] - 0.5) < 1e-16
    u = np.linspace(-6, 6, 101)
    assert np.allclose(orc.gelu_fwd(u) - orc.gelu_fwd(-u), u, atol=1e-14)   # u Phi(u) + u Phi(-u)... = u
    assert orc.relu_fwd(np.array([0.0]))[0] == 0 and orc.relu_bwd(np.array([1.0]), np.array([0.0]))[0] == 0


# ---------------------------------------------------------------- (5) library cross-check
@pytest.mark.parametrize("norm", ["post", "pre"])
@pytest.mark.parametrize("act", ["relu", "gelu"])
@pytest.mark.parametrize("masked", [False, True])
def test_against_torch_encoder_layer(norm, act, masked):
    torch = pytest.importorskip("torch")
    cfg = CFG1
    lengths = [13, 4] if masked else None
    inp = _inputs(cfg, seed=7, lengths=lengths)
    p, X, dY = inp["params"], inp["X"], inp["dY"]
    layer = torch.nn.TransformerEncoderLayer(cfg.D, cfg.H, cfg.F, dropout=0.0, activation=act,
                                             layer_norm_eps=cfg.eps, batch_first=True,
                                             norm_first=(norm == "pre"), dtype=torch.float64)
    layer.train()
    t = lambda a: torch.tensor(np.asarray(a, np.float64))
    with torch.no_grad():
        layer.self_attn.in_proj_weight.copy_(t(p["Wqkv"]))
        layer.self_attn.in_proj_bias.copy_(t(p["bqkv"]))
        layer.self_attn.out_proj.weight.copy_(t(p["Wo"]))
        layer.self_attn.out_proj.bias.copy_(t(p["bo"]))
        layer.linear1.weight.copy_(t(p["W1"]))
        layer.linear1.bias.copy_(t(p["b1"]))
        layer.linear2.weight.copy_(t(p["W2"]))
        layer.linear2.bias.copy_(t(p["b2"]))
        layer.norm1.weight.copy_(t(p["ln1_g"]))
        layer.norm1.bias.copy_(t(p["ln1_b"]))
        layer.norm2.weight.copy_(t(p["ln2_g"]))
        layer.norm2.bias.copy_(t(p["ln2_b"]))
    x = t(X).requires_grad_(True)
    mask = None
    if masked:
        mask = torch.arange(cfg.T)[None, :] >= torch.tensor(lengths)[:, None]
    y = layer(x, src_key_padding_mask=mask)
    (y * t(dY)).sum().backward()
    Y, dX, g = orc.layer_forward_backward(p, X, dY, inp["lengths"], heads=cfg.H, act=act, norm=norm, eps=cfg.eps)
    assert np.allclose(Y, y.detach().numpy(), atol=1e-11)
    assert np.allclose(dX, x.grad.numpy(), atol=1e-10)
    got = {"Wqkv": layer.self_attn.in_proj_weight.grad, "bqkv": layer.self_attn.in_proj_bias.grad,
           "Wo": layer.self_attn.out_proj.weight.grad, "bo": layer.self_attn.out_proj.bias.grad,
           "W1": layer.linear1.weight.grad, "b1": layer.linear1.bias.grad,
           "W2": layer.linear2.weight.grad, "b2": layer.linear2.bias.grad,
           "ln1_g": layer.norm1.weight.grad, "ln1_b": layer.norm1.bias.grad,
           "ln2_g": layer.norm2.weight.grad, "ln2_b": layer.norm2.bias.grad}
    for k in PARAM_NAMES:
        assert np.allclose(g[k], got[k].numpy(), atol=1e-10), k


# ---------------------------------------------------------------- (6) brute force, loops only
def _loops_forward(p, X, lengths, H, act, norm, eps, causal=False, masks=None):
    B, T, D = X.shape
    dh = D // H
    F = p["W1"].shape[0]

    def lin(x, W, b):
        return [sum(x[i] * W[o][i] for i in range(len(x))) + b[o] for o in range(len(b))]

    def ln(r, g, b):
        mu = sum(r) / len(r)
        var = sum((t - mu) ** 2 for t in r) / len(r)
        return [g[i] * (r[i] - mu) / math.sqrt(var + eps) + b[i] for i in range(len(r))]

    def actf(u):
        return max(u, 0.0) if act == "relu" else 0.5 * u * (1 + math.erf(u / math.sqrt(2)))

    mk = masks or {}
    keep = lambda name, *idx: 1.0 if mk.get(name) is None else float(mk[name][idx])
    Y = np.zeros((B, T, D))
    for b in range(B):
        n = T if lengths is None else int(lengths[b])
        xin = [list(map(float, X[b, t])) for t in range(T)]
        src = [ln(r, p["ln1_g"], p["ln1_b"]) for r in xin] if norm == "pre" else xin
        qkv = [lin(r, p["Wqkv"], p["bqkv"]) for r in src]
        O = [[0.0] * D for _ in range(T)]
        for h in range(H):
            for i in range(T):
                nk = min(n, i + 1) if causal else n          # keys this query may look at
                s = [sum(qkv[i][h * dh + d] * qkv[j][D + h * dh + d] for d in range(dh)) / math.sqrt(dh)
                     for j in range(nk)]
                m = max(s)
                e = [math.exp(v - m) for v in s]
                z = sum(e)
                for d in range(dh):
                    O[i][h * dh + d] = sum(e[j] / z * keep("attn", b, h, i, j) * qkv[j][2 * D + h * dh + d]
                                           for j in range(nk))
        for t in range(T):
            a = lin(O[t], p["Wo"], p["bo"])
            r1 = [xin[t][i] + a[i] * keep("proj", b, t, i) for i in range(D)]
            if norm == "post":
                y1 = ln(r1, p["ln1_g"], p["ln1_b"])
                f_in, skip = y1, y1
            else:
                f_in, skip = ln(r1, p["ln2_g"], p["ln2_b"]), r1
            u = lin(f_in, p["W1"], p["b1"])
            fo = lin([actf(v) * keep("ffn", b, t, k) for k, v in enumerate(u)], p["W2"], p["b2"])
            r2 = [skip[i] + fo[i] * keep("out", b, t, i) for i in range(D)]
            Y[b, t] = ln(r2, p["ln2_g"], p["ln2_b"]) if norm == "post" else r2
    return Y


@pytest.mark.parametrize("norm", ["post", "pre"])
@pytest.mark.parametrize("act", ["relu", "gelu"])
def test_against_scalar_loops(norm, act):
    cfg = CFG1.with_(B=2, T=3, D=4, H=2, F=8)
    inp = make_inputs(cfg, seed=9, nontrivial=True)
    p = {k: v.astype(np.float64) for k, v in inp["params"].items()}
    X = inp["X"].astype(np.float64)
    lengths = np.array([2, 3], np.int32)
    want = _loops_forward(p, X, lengths, cfg.H, act, norm, 1e-5)
    got, _ = orc.layer_forward(p, X, lengths, heads=cfg.H, act=act, norm=norm, eps=1e-5)
    assert np.allclose(got, want, atol=1e-13)


def test_stack_matches_chained_single_layers():
    from workloads import make_stack_inputs
    cfg = CFG1.with_(layers=3, norm="pre", act="gelu")
    inp = make_stack_inputs(cfg, seed=0, nontrivial=True)
    kw = dict(heads=cfg.H, act="gelu", norm="pre", eps=cfg.eps)
    Y, dX, grads = orc.stack_forward_backward(inp["params"], inp["X"], inp["dY"], None, **kw)
    x = inp["X"].astype(np.float64)
    caches = []
    for p in inp["params"]:
        x, c = orc.layer_forward(p, x, None, **kw)
        caches.append(c)
    assert np.array_equal(Y, x)
    d = inp["dY"].astype(np.float64)
    for l in (2, 1, 0):
        d, g = orc.layer_backward(inp["params"][l], caches[l], d)
        for k in PARAM_NAMES:
            assert np.array_equal(g[k], grads[l][k])
    assert np.array_equal(d, dX)


# ---------------------------------------------------------------- (8) the causal variant
@pytest.mark.parametrize("norm", ["post", "pre"])
def test_causal_against_scalar_loops(norm):
    cfg = CFG1.with_(B=2, T=5, D=4, H=2, F=8)
    inp = make_inputs(cfg, seed=10, nontrivial=True)
    p = {k: v.astype(np.float64) for k, v in inp["params"].items()}
    X = inp["X"].astype(np.float64)
    for lengths in (None, np.array([3, 5], np.int32)):
        want = _loops_forward(p, X, lengths, cfg.H, "gelu", norm, 1e-5, causal=True)
        got, _ = orc.layer_forward(p, X, lengths, heads=cfg.H, act="gelu", norm=norm, eps=1e-5, causal=True)
        assert np.allclose(got, want, atol=1e-13)
        plain, _ = orc.layer_forward(p, X, lengths, heads=cfg.H, act="gelu", norm=norm, eps=1e-5)
        assert not np.allclose(got, plain, atol=1e-3)          # the mask does something


@pytest.mark.parametrize("norm", ["post", "pre"])
@pytest.mark.parametrize("masked", [False, True])
def test_causal_against_torch_encoder_layer(norm, masked):
    """torch's encoder layer with a boolean upper-triangular src_mask (fp64), values and all gradients."""
    torch = pytest.importorskip("torch")
    cfg = CFG1
    lengths = [13, 4] if masked else None
    inp = _inputs(cfg, seed=8, lengths=lengths)
    p, X, dY = inp["params"], inp["X"], inp["dY"]
    layer = torch.nn.TransformerEncoderLayer(cfg.D, cfg.H, cfg.F, dropout=0.0, activation="gelu",
                                             layer_norm_eps=cfg.eps, batch_first=True,
                                             norm_first=(norm == "pre"), dtype=torch.float64)
    layer.train()
    t = lambda a: torch.tensor(np.asarray(a, np.float64))
    names = {"Wqkv": layer.self_attn.in_proj_weight, "bqkv": layer.self_attn.in_proj_bias,
             "Wo": layer.self_attn.out_proj.weight, "bo": layer.self_attn.out_proj.bias,
             "W1": layer.linear1.weight, "b1": layer.linear1.bias, "W2": layer.linear2.weight,
             "b2": layer.linear2.bias, "ln1_g": layer.norm1.weight, "ln1_b": layer.norm1.bias,
             "ln2_g": layer.norm2.weight, "ln2_b": layer.norm2.bias}
    with torch.no_grad():
        for k, w in names.items():
            w.copy_(t(p[k]))
    x = t(X).requires_grad_(True)
    future = torch.triu(torch.ones(cfg.T, cfg.T, dtype=torch.bool), diagonal=1)      # True = not allowed
    pad = None
    if masked:
        pad = torch.arange(cfg.T)[None, :] >= torch.tensor(lengths)[:, None]
    y = layer(x, src_mask=future, src_key_padding_mask=pad)
    (y * t(dY)).sum().backward()
    Y, dX, g = orc.layer_forward_backward(p, X, dY, inp["lengths"], heads=cfg.H, act="gelu", norm=norm,
                                          eps=cfg.eps, causal=True)
    assert np.allclose(Y, y.detach().numpy(), atol=1e-11)
    assert np.allclose(dX, x.grad.numpy(), atol=1e-10)
    for k, w in names.items():
        assert np.allclose(g[k], w.grad.numpy(), atol=1e-10), k


def test_causal_finite_differences():
    cfg = CFG1
    inp = _inputs(cfg, seed=5, lengths=[12, 7])
    kw = dict(heads=cfg.H, act="gelu", norm="post", eps=cfg.eps, causal=True)
    p = {k: v.astype(np.float64) for k, v in inp["params"].items()}
    X, dY, L = inp["X"].astype(np.float64), inp["dY"].astype(np.float64), inp["lengths"]
    _, dX, g = orc.layer_forward_backward(p, X, dY, L, **kw)
    rng = np.random.default_rng(12)
    h = 1e-6
    for name, arr, grad, n in [("X", X, dX, 60), ("Wqkv", p["Wqkv"], g["Wqkv"], 40), ("bqkv", p["bqkv"], g["bqkv"], 20),
                               ("Wo", p["Wo"], g["Wo"], 20)]:
        flat = arr.reshape(-1)
        scale = np.max(np.abs(grad)) + 1e-30
        for i in rng.choice(flat.size, size=min(n, flat.size), replace=False):
            old = flat[i]
            flat[i] = old + h
            lp = _loss(p, X, dY, L, kw)
            flat[i] = old - h
            lm = _loss(p, X, dY, L, kw)
            flat[i] = old
            assert abs((lp - lm) / (2 * h) - grad.reshape(-1)[i]) <= 2e-6 * scale, (name, int(i))


def test_causal_structure():
    """No information flows backwards in time; probabilities above the diagonal are exactly 0."""
    cfg = CFG1
    inp = _inputs(cfg, seed=6, lengths=[16, 9])
    p, X, dY, L = inp["params"], inp["X"].astype(np.float64), inp["dY"].astype(np.float64), inp["lengths"]
    kw = dict(heads=cfg.H, act="relu", norm="pre", eps=cfg.eps, causal=True)
    Y, c = orc.layer_forward(p, X, L, **kw)
    P = c["attn"]["P"]
    iu = np.triu_indices(cfg.T, k=1)
    assert np.all(P[:, :, iu[0], iu[1]] == 0.0)
    assert np.allclose(P.sum(-1), 1.0, atol=1e-14)
    assert np.all(P[1, :, :, 9:] == 0.0)                        # padding keys stay masked too
    assert np.allclose(P[:, :, 0, 0], 1.0)                      # the first query sees only itself
    t0 = 6
    X2 = X.copy()
    X2[:, t0:] += np.random.default_rng(0).standard_normal(X2[:, t0:].shape)
    Y2, _ = orc.layer_forward(p, X2, L, **kw)
    assert np.array_equal(Y2[:, :t0], Y[:, :t0])                # earlier positions do not see the change
    assert not np.allclose(Y2[:, t0:], Y[:, t0:])
    # and the gradient of early outputs w.r.t. later inputs is zero
    dY0 = dY.copy()
    dY0[:, t0:] = 0.0
    _, dX, _ = orc.layer_forward_backward(p, X, dY0, L, **kw)
    assert np.all(dX[:, t0:] == 0.0) and np.any(dX[:, :t0] != 0.0)
    # a single-token sequence is unaffected by the causal mask
    cfg1 = CFG1.with_(T=1)
    inp1 = make_inputs(cfg1, seed=2, nontrivial=True)
    a, _ = orc.layer_forward(inp1["params"], inp1["X"], None, heads=cfg1.H, act="relu", norm="post", eps=cfg1.eps)
    b_, _ = orc.layer_forward(inp1["params"], inp1["X"], None, heads=cfg1.H, act="relu", norm="post", eps=cfg1.eps,
                              causal=True)
    assert np.array_equal(a, b_)

"""CPU oracle for one Transformer encoder layer, forward and backward, in float64.

TEST INFRASTRUCTURE ONLY.  This file is the yardstick the HIP library is
measured against: it is imported by the tests, by the smoke check and by the
benchmark's CPU-baseline leg, and by nothing on the product path.  It shares no
code with the HIP implementation and imports nothing from it.

What it computes.  The paper (Flashlight, arXiv 2201.12465) only *names* the
architectures whose training step it benchmarks -- Transformers, BERT-like
language models, ViT, the ASR Transformer (Section 3 "Principles", Section 4.3
"Packages and Applications", Section 5.1.2 Table 3) -- and describes how they
execute: every operator is a composition of tensor primitives (Section 4.1.1;
ReLU is the max primitive), recorded on a tape and differentiated by
per-operator gradient functions that add into their inputs' gradients
(Section 4.2 "Automatic Differentiation", the cosine-operator listing).  It
gives no equations for the layer, so the oracle is the textbook definition of
a multi-head self-attention encoder layer written out step by step, and the
backward pass is the chain rule applied to each of those steps in reverse, one
gradient function per forward step, accumulating into inputs that are used
twice (the residual connections) -- the same structure as the paper's tape.

Conventions fixed where the paper is silent (each is listed in the design
notes of the repository):
  * weights are [out, in]; a linear map is  y = x W^T + b;
    Wqkv = [Wq; Wk; Wv] stacked on rows; head h owns columns h*dh..(h+1)*dh;
  * scores are (q . k) / sqrt(dh); key j of sequence b is masked out iff
    j >= lengths[b] (score -inf before the softmax, probability exactly 0);
    padded *query* rows are ordinary rows;
  * the causal variant (the autoregressive language-model task named in Section 4.3
    "Text") additionally masks out key j for query i iff j > i; with lengths >= 1 every
    query keeps at least key 0;
  * LayerNorm uses the biased variance and eps inside the square root;
  * GELU is the exact erf form; relu'(0) = 0;
  * dropout is off unless the caller passes `masks` (the four scaled keep masks of
    oracle/dropout.py: attention probabilities after the softmax, the attention
    projection's output and the second feed-forward linear's output before their
    residual adds, the feed-forward activation's output); the softmax itself and its
    backward rule are unchanged, the mask multiplies P on the way to P V.

Every function works on float64 numpy arrays; inputs of other dtypes are
promoted.  Parity pins live in tests/test_oracle_*.py.
"""
from __future__ import annotations

import math
import numpy as np

try:  # vectorised erf; the fallback is slow but exact enough (libm erf)
    from scipy.special import erf as _erf
except Exception:  # pragma: no cover
    _erf = np.vectorize(math.erf, otypes=[np.float64])

_SQRT2 = math.sqrt(2.0)
_INV_SQRT_2PI = 1.0 / math.sqrt(2.0 * math.pi)


def _f64(a):
    return np.asarray(a, dtype=np.float64)


# ----------------------------------------------------------------------------
# primitives: each forward step and the gradient function of that step
# ----------------------------------------------------------------------------

def linear_fwd(x, W, b):
    """y[m, o] = sum_i x[m, i] W[o, i] + b[o]   (matmul + add primitives, Section 4.1.1)."""
    return _f64(x) @ _f64(W).T + _f64(b)


def linear_bwd(dy, x, W):
    """Gradient function of linear_fwd: dx = dy W, dW = dy^T x, db = column sums of dy."""
    dy, x, W = _f64(dy), _f64(x), _f64(W)
    dy2 = dy.reshape(-1, dy.shape[-1])
    x2 = x.reshape(-1, x.shape[-1])
    return dy @ W, dy2.T @ x2, dy2.sum(axis=0)


def relu_fwd(u):
    """ReLU through the max primitive (Section 4.1.1): relu(0) = 0."""
    return np.maximum(_f64(u), 0.0)


def relu_bwd(dg, u):
    return _f64(dg) * (_f64(u) > 0.0)


def gelu_fwd(u):
    """Exact GELU: u * Phi(u), Phi the standard normal CDF."""
    u = _f64(u)
    return 0.5 * u * (1.0 + _erf(u / _SQRT2))


def gelu_bwd(dg, u):
    """d/du [u Phi(u)] = Phi(u) + u phi(u)."""
    u = _f64(u)
    cdf = 0.5 * (1.0 + _erf(u / _SQRT2))
    pdf = _INV_SQRT_2PI * np.exp(-0.5 * u * u)
    return _f64(dg) * (cdf + u * pdf)


def act_fwd(u, act):
    return relu_fwd(u) if act == "relu" else gelu_fwd(u)


def act_bwd(dg, u, act):
    return relu_bwd(dg, u) if act == "relu" else gelu_bwd(dg, u)


def layernorm_fwd(x, gamma, beta, eps):
    """Per row over the last axis: xhat = (x - mean) / sqrt(var + eps), y = gamma xhat + beta.

    var is the biased (divide by D) variance.  Returns y, xhat, rstd ([..., 1]).
    """
    x = _f64(x)
    mu = x.mean(axis=-1, keepdims=True)
    xc = x - mu
    var = (xc * xc).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = xc * rstd
    return _f64(gamma) * xhat + _f64(beta), xhat, rstd


def layernorm_bwd(dy, xhat, rstd, gamma):
    """Gradient function of layernorm_fwd.

    With g = dy * gamma:  dx = rstd * (g - mean(g) - xhat * mean(g * xhat)),
    dgamma = sum over rows of dy * xhat, dbeta = sum over rows of dy.
    """
    dy, xhat = _f64(dy), _f64(xhat)
    g = dy * _f64(gamma)
    m1 = g.mean(axis=-1, keepdims=True)
    m2 = (g * xhat).mean(axis=-1, keepdims=True)
    dx = rstd * (g - m1 - xhat * m2)
    D = dy.shape[-1]
    dgamma = (dy * xhat).reshape(-1, D).sum(axis=0)
    dbeta = dy.reshape(-1, D).sum(axis=0)
    return dx, dgamma, dbeta


def split_heads(a, H):
    """[B, T, D] -> [B, H, T, dh]; head h is columns h*dh..(h+1)*dh."""
    B, T, D = a.shape
    return a.reshape(B, T, H, D // H).transpose(0, 2, 1, 3)


def merge_heads(a):
    """[B, H, T, dh] -> [B, T, H*dh]."""
    B, H, T, dh = a.shape
    return a.transpose(0, 2, 1, 3).reshape(B, T, H * dh)


def key_mask(lengths, B, T):
    """Boolean [B, T]: True where key j of sequence b is padding (j >= lengths[b])."""
    if lengths is None:
        return np.zeros((B, T), dtype=bool)
    lengths = np.asarray(lengths).astype(np.int64)
    if lengths.shape != (B,) or np.any(lengths < 1) or np.any(lengths > T):
        raise ValueError("lengths must be B integers in [1, T]")
    return np.arange(T)[None, :] >= lengths[:, None]


def attention_fwd(Q, K, V, lengths=None, causal=False, keep=None):
    """Masked scaled-dot-product attention.  Q, K, V: [B, H, T, dh].
    keep (optional, [B, H, T, T]): scaled dropout keep mask; then O = (P * keep) V, P is returned undropped.

    S = Q K^T / sqrt(dh); masked keys get -inf; P = softmax over keys; O = P V.
    Masked: padding keys (j >= lengths[b]) and, if causal, keys after the query (j > i).
    Returns O [B, H, T, dh] and P [B, H, T, T].
    """
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    B, H, T, dh = Q.shape
    S = (Q @ K.transpose(0, 1, 3, 2)) / math.sqrt(dh)
    pad = key_mask(lengths, B, T)
    S = np.where(pad[:, None, None, :], -np.inf, S)
    if causal:
        future = np.arange(T)[None, :] > np.arange(T)[:, None]      # [query i, key j]: j > i
        S = np.where(future[None, None, :, :], -np.inf, S)
    S = S - S.max(axis=-1, keepdims=True)
    E = np.exp(S)
    P = E / E.sum(axis=-1, keepdims=True)
    return (P if keep is None else P * _f64(keep)) @ V, P


def attention_bwd(dO, Q, K, V, P, keep=None):
    """Gradient function of attention_fwd.

    dV = P^T dO;  dP = dO V^T;  dS = P * (dP - rowsum(dP * P));
    dQ = dS K / sqrt(dh);  dK = dS^T Q / sqrt(dh).
    Masked keys have P = 0, hence dS = 0 there and zero rows in dK, dV.
    With a dropout keep mask the forward used Pd = P * keep:  dV = Pd^T dO and dP = (dO V^T) * keep.
    """
    dO, Q, K, V, P = map(_f64, (dO, Q, K, V, P))
    dh = Q.shape[-1]
    Pd = P if keep is None else P * _f64(keep)
    dV = Pd.transpose(0, 1, 3, 2) @ dO
    dP = dO @ V.transpose(0, 1, 3, 2)
    if keep is not None:
        dP = dP * _f64(keep)
    dS = P * (dP - (dP * P).sum(axis=-1, keepdims=True))
    scale = 1.0 / math.sqrt(dh)
    dQ = (dS @ K) * scale
    dK = (dS.transpose(0, 1, 3, 2) @ Q) * scale
    return dQ, dK, dV


# ----------------------------------------------------------------------------
# the layer
# ----------------------------------------------------------------------------

def _self_attention_fwd(x, p, H, lengths, causal=False, keep=None):
    D = x.shape[-1]
    qkv = linear_fwd(x, p["Wqkv"], p["bqkv"])
    Q = split_heads(qkv[..., :D], H)
    K = split_heads(qkv[..., D:2 * D], H)
    V = split_heads(qkv[..., 2 * D:], H)
    Oh, P = attention_fwd(Q, K, V, lengths, causal, keep)
    O = merge_heads(Oh)
    A = linear_fwd(O, p["Wo"], p["bo"])
    return A, dict(x=x, Q=Q, K=K, V=V, P=P, O=O, keep=keep)


def _self_attention_bwd(dA, p, c, g):
    """Adds dWo, dbo, dWqkv, dbqkv to g and returns the gradient w.r.t. the block's input."""
    dO, g["Wo"], g["bo"] = linear_bwd(dA, c["O"], p["Wo"])
    H = c["Q"].shape[1]
    dQ, dK, dV = attention_bwd(split_heads(dO, H), c["Q"], c["K"], c["V"], c["P"], c.get("keep"))
    dqkv = np.concatenate([merge_heads(dQ), merge_heads(dK), merge_heads(dV)], axis=-1)
    dx, g["Wqkv"], g["bqkv"] = linear_bwd(dqkv, c["x"], p["Wqkv"])
    return dx


def _ffn_fwd(x, p, act, keep=None):
    """keep (optional): scaled dropout keep mask on the activation's output; G is what the second linear reads."""
    U = linear_fwd(x, p["W1"], p["b1"])
    G = act_fwd(U, act)
    if keep is not None:
        G = G * _f64(keep)
    Fo = linear_fwd(G, p["W2"], p["b2"])
    return Fo, dict(x=x, U=U, G=G, keep=keep)


def _ffn_bwd(dFo, p, c, act, g):
    dG, g["W2"], g["b2"] = linear_bwd(dFo, c["G"], p["W2"])
    if c.get("keep") is not None:
        dG = dG * _f64(c["keep"])
    dU = act_bwd(dG, c["U"], act)
    dx, g["W1"], g["b1"] = linear_bwd(dU, c["x"], p["W1"])
    return dx


def layer_forward(params, X, lengths=None, *, heads, act="relu", norm="post", eps=1e-5, causal=False, masks=None):
    """Forward pass.  X: [B, T, D].  Returns (Y, cache).  causal: query i attends to keys j <= i only.
    masks: None (no dropout) or the dict of scaled keep masks "attn", "proj", "ffn", "out".

    post-LN:  Y1 = LN1(X + Attn(X));   Y = LN2(Y1 + FFN(Y1))
    pre-LN:   R1 = X + Attn(LN1(X));   Y = R1 + FFN(LN2(R1))
    With dropout, Attn(.) and FFN(.) stand for the dropped-out branch outputs (keep masks "proj" and
    "out" applied right before the residual adds).
    """
    p = {k: _f64(v) for k, v in params.items()}
    X = _f64(X)
    mk = masks or {}
    ka, kp, kf, ko = (None if mk.get(k) is None else _f64(mk[k]) for k in ("attn", "proj", "ffn", "out"))
    drop = lambda a, k: a if k is None else a * k
    c = {"act": act, "norm": norm, "keep_proj": kp, "keep_out": ko}
    if norm == "post":
        A, c["attn"] = _self_attention_fwd(X, p, heads, lengths, causal, ka)
        R1 = X + drop(A, kp)
        Y1, c["xhat1"], c["rstd1"] = layernorm_fwd(R1, p["ln1_g"], p["ln1_b"], eps)
        Fo, c["ffn"] = _ffn_fwd(Y1, p, act, kf)
        R2 = Y1 + drop(Fo, ko)
        Y, c["xhat2"], c["rstd2"] = layernorm_fwd(R2, p["ln2_g"], p["ln2_b"], eps)
    elif norm == "pre":
        N1, c["xhat1"], c["rstd1"] = layernorm_fwd(X, p["ln1_g"], p["ln1_b"], eps)
        A, c["attn"] = _self_attention_fwd(N1, p, heads, lengths, causal, ka)
        R1 = X + drop(A, kp)
        N2, c["xhat2"], c["rstd2"] = layernorm_fwd(R1, p["ln2_g"], p["ln2_b"], eps)
        Fo, c["ffn"] = _ffn_fwd(N2, p, act, kf)
        Y = R1 + drop(Fo, ko)
    else:
        raise ValueError(norm)
    return Y, c


def layer_backward(params, cache, dY):
    """Backward pass given the upstream gradient dY.  Returns (dX, grads dict of 12 arrays)."""
    p = {k: _f64(v) for k, v in params.items()}
    c, dY, g = cache, _f64(dY), {}
    act = c["act"]
    # the gradient that enters a dropped-out branch is the residual sum's gradient times the keep mask
    drop = lambda a, k: a if k is None else a * k
    kp, ko = c.get("keep_proj"), c.get("keep_out")
    if c["norm"] == "post":
        dR2, g["ln2_g"], g["ln2_b"] = layernorm_bwd(dY, c["xhat2"], c["rstd2"], p["ln2_g"])
        dY1 = dR2 + _ffn_bwd(drop(dR2, ko), p, c["ffn"], act, g)          # Y1 feeds the residual and the FFN
        dR1, g["ln1_g"], g["ln1_b"] = layernorm_bwd(dY1, c["xhat1"], c["rstd1"], p["ln1_g"])
        dX = dR1 + _self_attention_bwd(drop(dR1, kp), p, c["attn"], g)    # X feeds the residual and attention
    else:
        dN2 = _ffn_bwd(drop(dY, ko), p, c["ffn"], act, g)
        dR1_ln, g["ln2_g"], g["ln2_b"] = layernorm_bwd(dN2, c["xhat2"], c["rstd2"], p["ln2_g"])
        dR1 = dY + dR1_ln
        dN1 = _self_attention_bwd(drop(dR1, kp), p, c["attn"], g)
        dX_ln, g["ln1_g"], g["ln1_b"] = layernorm_bwd(dN1, c["xhat1"], c["rstd1"], p["ln1_g"])
        dX = dR1 + dX_ln
    return dX, g


def layer_forward_backward(params, X, dY, lengths=None, **kw):
    """Convenience: (Y, dX, grads)."""
    Y, c = layer_forward(params, X, lengths, **kw)
    dX, g = layer_backward(params, c, dY)
    return Y, dX, g


def stack_forward_backward(param_list, X, dY, lengths=None, **kw):
    """L layers chained through the same layer function.

    Keeps only each layer's input during the forward sweep and recomputes the
    layer's intermediates when its turn comes in the backward sweep, to bound
    memory.  Returns (Y, dX, [grads per layer]).
    """
    xs = [_f64(X)]
    for p in param_list:
        y, _ = layer_forward(p, xs[-1], lengths, **kw)
        xs.append(y)
    Y = xs[-1]
    d = _f64(dY)
    grads = [None] * len(param_list)
    for l in reversed(range(len(param_list))):
        _, c = layer_forward(param_list[l], xs[l], lengths, **kw)
        d, grads[l] = layer_backward(param_list[l], c, d)
    return Y, d, grads

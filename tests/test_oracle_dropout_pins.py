"""Pins for the oracle's dropout: the generator against its published known-answer vectors and a
scalar re-implementation, the mask conventions, and the layer with masks against scalar loops,
finite differences and torch's encoder layer with its dropout modules replaced by fixed masks."""
import math
import os

import numpy as np
import pytest

from oracle import dropout as odr
from oracle import oracle as orc
from test_oracle_pins import CFG1, _inputs, _loops_forward
from workloads import PARAM_NAMES, make_inputs

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "philox4x32_10_kat.txt")


def _scalar_philox(c, k):
    """Philox4x32-10 on Python integers, straight from the round description in the SC'11 paper."""
    c, k = list(c), list(k)
    for _ in range(10):
        p0, p1 = 0xD2511F53 * c[0], 0xCD9E8D57 * c[2]
        c = [(p1 >> 32) ^ c[1] ^ k[0], p1 & 0xFFFFFFFF, (p0 >> 32) ^ c[3] ^ k[1], p0 & 0xFFFFFFFF]
        k = [(k[0] + 0x9E3779B9) & 0xFFFFFFFF, (k[1] + 0xBB67AE85) & 0xFFFFFFFF]
    return c


def test_philox_known_answers():
    rows = [l.split() for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        v = [int(x, 16) for x in r]
        got = odr.philox4x32_10(tuple(np.uint32(x) for x in v[:4]), (v[4], v[5]))
        assert [int(np.asarray(g).reshape(-1)[0]) for g in got] == v[6:]
        assert _scalar_philox(v[:4], v[4:6]) == v[6:]


def test_philox_vectorised_equals_scalar():
    rng = np.random.default_rng(0)
    c = rng.integers(0, 2 ** 32, size=(4, 50), dtype=np.uint64).astype(np.uint32)
    key = (0x12345678, 0x9ABCDEF0)
    got = odr.philox4x32_10(tuple(c), key)
    for i in range(50):
        assert [int(g[i]) for g in got] == _scalar_philox([int(x) for x in c[:, i]], key)


def test_mask_conventions():
    seed = (0xDEADBEEF << 32) | 0x01234567
    key = (0x01234567, 0xDEADBEEF)
    p = 0.3
    thr = odr.threshold(p)
    assert thr == int(math.floor(0.3 * 2 ** 32)) and odr.threshold(0.0) == 0
    m = odr.keep_mask_rows(7, 13, 3, p, seed)
    for row in range(7):
        for n in range(13):
            w = _scalar_philox([n // 4, row, 3, 0], key)[n % 4]
            assert m[row, n] == (1.0 / (1.0 - p) if w >= thr else 0.0)
    a = odr.keep_mask_attention(2, 3, 9, p, seed)
    for (b, h, i, j) in [(0, 0, 0, 0), (1, 2, 8, 7), (0, 1, 4, 5), (1, 0, 3, 3)]:
        w = _scalar_philox([j // 4, i, 1, b * 3 + h], key)[j % 4]
        assert a[b, h, i, j] == (1.0 / (1.0 - p) if w >= thr else 0.0)
    assert np.array_equal(odr.keep_mask_rows(5, 8, 2, 0.0, seed), np.ones((5, 8)))
    with pytest.raises(ValueError):
        odr.threshold(1.0)


def test_mask_statistics_and_independence():
    p, seed = 0.1, 42
    m = odr.keep_mask_rows(512, 768, 2, p, seed)
    kept = m != 0
    n = kept.size
    assert abs(kept.mean() - (1 - p)) < 5 * math.sqrt(p * (1 - p) / n)
    assert np.allclose(m[kept], 1 / (1 - p)) and abs(m.mean() - 1.0) < 5e-3
    assert np.array_equal(m, odr.keep_mask_rows(512, 768, 2, p, seed))                  # deterministic
    for other in (odr.keep_mask_rows(512, 768, 4, p, seed), odr.keep_mask_rows(512, 768, 2, p, seed + 1)):
        agree = ((other != 0) == kept).mean()                                           # independent masks agree
        assert abs(agree - ((1 - p) ** 2 + p ** 2)) < 5e-3                               # with prob. (1-p)^2 + p^2
    # neighbouring elements are uncorrelated
    c = np.corrcoef(kept[:, :-1].ravel(), kept[:, 1:].ravel())[0, 1]
    assert abs(c) < 1e-2


def _masks(cfg, p_attn, p_hidden, seed):
    return odr.layer_masks(cfg.B, cfg.T, cfg.D, cfg.H, cfg.F, p_attn, p_hidden, seed)


def test_all_ones_masks_are_no_dropout():
    cfg = CFG1
    inp = _inputs(cfg, seed=1, lengths=[16, 7])
    kw = dict(heads=cfg.H, act="gelu", norm="post", eps=cfg.eps)
    a = orc.layer_forward_backward(inp["params"], inp["X"], inp["dY"], inp["lengths"], **kw)
    b = orc.layer_forward_backward(inp["params"], inp["X"], inp["dY"], inp["lengths"], masks=_masks(cfg, 0.0, 0.0, 5),
                                   **kw)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    for k in PARAM_NAMES:
        assert np.array_equal(a[2][k], b[2][k])


@pytest.mark.parametrize("norm", ["post", "pre"])
@pytest.mark.parametrize("causal", [False, True])
def test_dropout_against_scalar_loops(norm, causal):
    cfg = CFG1.with_(B=2, T=5, D=8, H=2, F=12)
    inp = make_inputs(cfg, seed=13, nontrivial=True)
    p = {k: v.astype(np.float64) for k, v in inp["params"].items()}
    X = inp["X"].astype(np.float64)
    lengths = np.array([4, 5], np.int32)
    masks = _masks(cfg, 0.25, 0.4, seed=77)
    want = _loops_forward(p, X, lengths, cfg.H, "gelu", norm, 1e-5, causal=causal, masks=masks)
    got, _ = orc.layer_forward(p, X, lengths, heads=cfg.H, act="gelu", norm=norm, eps=1e-5, causal=causal, masks=masks)
    assert np.allclose(got, want, atol=1e-13)
    plain, _ = orc.layer_forward(p, X, lengths, heads=cfg.H, act="gelu", norm=norm, eps=1e-5, causal=causal)
    assert not np.allclose(got, plain, atol=1e-3)


@pytest.mark.parametrize("norm,act", [("post", "gelu"), ("pre", "relu")])
def test_dropout_finite_differences(norm, act):
    """With the masks held fixed the layer is a smooth function of its inputs: central differences."""
    cfg = CFG1
    inp = _inputs(cfg, seed=21, lengths=[15, 6])
    masks = _masks(cfg, 0.2, 0.3, seed=9)
    kw = dict(heads=cfg.H, act=act, norm=norm, eps=cfg.eps, masks=masks)
    p = {k: v.astype(np.float64) for k, v in inp["params"].items()}
    X, dY, L = inp["X"].astype(np.float64), inp["dY"].astype(np.float64), inp["lengths"]
    _, dX, g = orc.layer_forward_backward(p, X, dY, L, **kw)
    _, cache = orc.layer_forward(p, X, L, **kw)
    assert act == "gelu" or np.min(np.abs(cache["ffn"]["U"])) > 1e-5
    rng = np.random.default_rng(3)
    h = 1e-6
    loss = lambda: float(np.sum(orc.layer_forward(p, X, L, **kw)[0] * dY))
    for name, arr, grad, n in [("X", X, dX, 50)] + [(k, p[k], g[k], 16) for k in PARAM_NAMES]:
        flat = arr.reshape(-1)
        scale = np.max(np.abs(grad)) + 1e-30
        for i in rng.choice(flat.size, size=min(n, flat.size), replace=False):
            old = flat[i]
            flat[i] = old + h
            lp = loss()
            flat[i] = old - h
            lm = loss()
            flat[i] = old
            assert abs((lp - lm) / (2 * h) - grad.reshape(-1)[i]) <= 2e-6 * scale, (name, int(i))


@pytest.mark.parametrize("norm", ["post", "pre"])
def test_hidden_dropout_sites_against_torch(norm):
    """torch's encoder layer with its three Dropout modules replaced by multiplications with the
    oracle's masks (attention dropout off: torch draws that one internally): placement of the three
    hidden-state sites relative to residuals and LayerNorms, values and all gradients, fp64."""
    torch = pytest.importorskip("torch")
    cfg = CFG1
    inp = _inputs(cfg, seed=17, lengths=[13, 4])
    p, X, dY = inp["params"], inp["X"], inp["dY"]
    masks = _masks(cfg, 0.0, 0.35, seed=123)
    layer = torch.nn.TransformerEncoderLayer(cfg.D, cfg.H, cfg.F, dropout=0.0, activation="gelu",
                                             layer_norm_eps=cfg.eps, batch_first=True,
                                             norm_first=(norm == "pre"), dtype=torch.float64)
    layer.train()
    t = lambda a: torch.tensor(np.asarray(a, np.float64))

    class Fixed(torch.nn.Module):
        def __init__(self, m):
            super().__init__()
            self.m = t(m)

        def forward(self, x):
            return x * self.m

    layer.dropout1, layer.dropout, layer.dropout2 = Fixed(masks["proj"]), Fixed(masks["ffn"]), Fixed(masks["out"])
    names = {"Wqkv": layer.self_attn.in_proj_weight, "bqkv": layer.self_attn.in_proj_bias,
             "Wo": layer.self_attn.out_proj.weight, "bo": layer.self_attn.out_proj.bias,
             "W1": layer.linear1.weight, "b1": layer.linear1.bias, "W2": layer.linear2.weight,
             "b2": layer.linear2.bias, "ln1_g": layer.norm1.weight, "ln1_b": layer.norm1.bias,
             "ln2_g": layer.norm2.weight, "ln2_b": layer.norm2.bias}
    with torch.no_grad():
        for k, w in names.items():
            w.copy_(t(p[k]))
    x = t(X).requires_grad_(True)
    pad = torch.arange(cfg.T)[None, :] >= torch.tensor([13, 4])[:, None]
    y = layer(x, src_key_padding_mask=pad)
    (y * t(dY)).sum().backward()
    Y, dX, g = orc.layer_forward_backward(p, X, dY, inp["lengths"], heads=cfg.H, act="gelu", norm=norm, eps=cfg.eps,
                                          masks=masks)
    assert np.allclose(Y, y.detach().numpy(), atol=1e-11)
    assert np.allclose(dX, x.grad.numpy(), atol=1e-10)
    for k, w in names.items():
        assert np.allclose(g[k], w.grad.numpy(), atol=1e-10), k


def test_attention_dropout_definition():
    """O = (P * keep) V with P the undropped softmax; dropped pairs pass no gradient to V or the scores."""
    rng = np.random.default_rng(5)
    B, H, T, dh = 1, 2, 6, 4
    Q, K, V, dO = (rng.standard_normal((B, H, T, dh)) for _ in range(4))
    keep = odr.keep_mask_attention(B, H, T, 0.5, seed=3)
    O, P = orc.attention_fwd(Q, K, V, None, False, keep)
    assert np.allclose(P.sum(-1), 1.0)
    for h in range(H):
        for i in range(T):
            want = sum(P[0, h, i, j] * keep[0, h, i, j] * V[0, h, j] for j in range(T))
            assert np.allclose(O[0, h, i], want, atol=1e-14)
    dQ, dK, dV = orc.attention_bwd(dO, Q, K, V, P, keep)
    h_ = 1e-6
    for arr, grad in ((Q, dQ), (K, dK), (V, dV)):
        flat = arr.reshape(-1)
        for i in rng.choice(flat.size, 12, replace=False):
            old = flat[i]
            flat[i] = old + h_
            lp = np.sum(orc.attention_fwd(Q, K, V, None, False, keep)[0] * dO)
            flat[i] = old - h_
            lm = np.sum(orc.attention_fwd(Q, K, V, None, False, keep)[0] * dO)
            flat[i] = old
            assert abs((lp - lm) / (2 * h_) - grad.reshape(-1)[i]) < 1e-7

"""The allocation-free entry point fl_layer_forward_static against fl_layer_forward: two calls in a row
through the C ABI, the second with a smaller input, outputs compared bit for bit (same kernels) and, for
good measure, against the oracle at the layer tolerance; the caching allocator must not move."""
import numpy as np
import pytest

from oracle import oracle as orc
from gpu_util import BF16_TOL, F32_TOL, empty_dev, rel_err, stream_ptr, to_dev, to_np, torch_mod
from workloads import CONFIGS, make_inputs

pytestmark = pytest.mark.gpu


def _forward(cfg, inp, static, layer):
    torch = torch_mod()
    dt = cfg.dtype
    p = {k: to_dev(v, dt) for k, v in inp["params"].items()}
    X = to_dev(inp["X"], dt)
    Y = empty_dev(X.shape, dt)
    L = torch.tensor(inp["lengths"], dtype=torch.int32, device="cuda") if inp["lengths"] is not None else None
    if static:
        layer.forward_static(p, X, L, cfg.B, cfg.T, Y, stream_ptr())
    else:
        layer.forward(p, X, L, cfg.B, cfg.T, Y, stream_ptr())
    torch.cuda.synchronize()
    return to_np(Y)


@pytest.mark.parametrize("base,kw", [
    ("cfg3_bert_base_bf16", dict(B=6)),                                        # post-LN, GELU, key-padding mask
    ("cfg5_vit_b16_bf16", dict(B=5, layers=1)),                                # pre-LN, GELU, no mask, T = 197
    ("cfg2_small_f32", dict(B=3, T=70, D=128, H=2, F=264, causal=True)),       # fp32, ReLU, ragged tiles, causal
])
def test_static_forward_matches_forward_on_two_calls_in_a_row(base, kw):
    from paper_2201_12465_amd import binding as b
    cfg = CONFIGS[base].with_(**kw)
    small = cfg.with_(B=max(1, cfg.B // 2), T=cfg.T - 13,
                      len_lo=min(cfg.len_lo, cfg.T - 13), len_hi=min(cfg.len_hi, cfg.T - 13))
    layer = b.Layer(cfg.B, cfg.T, cfg.D, cfg.H, cfg.F, cfg.act, cfg.norm, cfg.dtype, cfg.eps, cfg.causal)
    plain = b.Layer(cfg.B, cfg.T, cfg.D, cfg.H, cfg.F, cfg.act, cfg.norm, cfg.dtype, cfg.eps, cfg.causal)
    tol = F32_TOL if cfg.dtype == "f32" else BF16_TOL
    try:
        for c, seed in ((cfg, 3), (small, 4)):          # the second call: fewer sequences, shorter ones
            inp = make_inputs(c, seed=seed, nontrivial=True)
            want = _forward(c, inp, False, plain)   # records a tape, which its next forward drops
            before = b.alloc_stats()
            got = _forward(c, inp, True, layer)
            after = b.alloc_stats()
            assert np.array_equal(got, want), (c.B, c.T)
            for k in ("backing_mallocs", "cache_hits", "cache_misses", "live_bytes"):
                assert after[k] == before[k], k       # nothing was taken from the caching allocator either
            ref, _ = orc.layer_forward(inp["params"], inp["X"], inp["lengths"], heads=c.H, act=c.act, norm=c.norm,
                                       eps=c.eps, causal=c.causal)
            assert rel_err(got, ref) <= tol
    finally:
        layer.destroy()
        plain.destroy()


def test_static_forward_rejects_what_does_not_fit():
    """Sizes beyond the static array's capacity are refused with a clear error before anything is enqueued;
    the handle stays usable."""
    from paper_2201_12465_amd import binding as b
    cfg = CONFIGS["cfg2_small_f32"]
    layer = b.Layer(64, 4096, cfg.D, cfg.H, cfg.F, cfg.act, cfg.norm, cfg.dtype, cfg.eps)
    inp = make_inputs(cfg, seed=0)
    p = {k: to_dev(v, cfg.dtype) for k, v in inp["params"].items()}
    big = empty_dev((64, 4096, cfg.D), cfg.dtype)          # 262144 tokens: far more than the array holds
    with pytest.raises(b.FlError) as e:
        layer.forward_static(p, big, None, 64, 4096, big, stream_ptr())
    assert e.value.status == b.FL_ERR_UNSUPPORTED and "static scratch" in str(e.value)
    X = to_dev(inp["X"], cfg.dtype)
    Y, Y2 = empty_dev(X.shape, cfg.dtype), empty_dev(X.shape, cfg.dtype)
    layer.forward_static(p, X, None, cfg.B, cfg.T, Y, stream_ptr())
    layer.forward(p, X, None, cfg.B, cfg.T, Y2, stream_ptr())
    with pytest.raises(b.FlError) as e:                     # a recorded forward is pending on the handle
        layer.forward_static(p, X, None, cfg.B, cfg.T, Y, stream_ptr())
    assert e.value.status == b.FL_ERR_STATE
    torch_mod().cuda.synchronize()
    assert np.array_equal(to_np(Y), to_np(Y2))
    layer.destroy()

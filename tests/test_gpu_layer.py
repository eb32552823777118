"""Layer-level parity: fl_layer_forward / fl_layer_backward through the C ABI
against the fp64 CPU oracle, on the seeded synthetic workloads.  Compared: Y, dX
and all 12 parameter gradients, each as max|gpu-ref| / max|ref|."""
import numpy as np
import pytest

from oracle import oracle as orc
from gpu_util import (BF16_TOL, F32_TOL, empty_dev, log_errors, rel_err, rel_err_l2, stream_ptr, to_dev, to_np,
                      torch_mod)
from workloads import CONFIGS, PARAM_NAMES, make_inputs, make_stack_inputs

pytestmark = pytest.mark.gpu


def run_layer_gpu(cfg, inp, layer=None, keep=False, dropout=None, peek_act=False):
    """dropout: None or (p_attn, p_hidden, seed).  peek_act: the layer runs on the test build of the library
    and the feed-forward activation's output, as the recorded forward holds it, is returned as a fourth value."""
    from paper_2201_12465_amd import binding as b
    torch = torch_mod()
    dt = cfg.dtype
    own = layer is None
    if own:
        layer = b.Layer(cfg.B, cfg.T, cfg.D, cfg.H, cfg.F, cfg.act, cfg.norm, dt, cfg.eps, cfg.causal,
                        L=b.test_lib() if peek_act else None)
    if dropout is not None:
        layer.set_dropout(*dropout)
    p = {k: to_dev(v, dt) for k, v in inp["params"].items()}
    g = {k: empty_dev(v.shape, dt) for k, v in inp["params"].items()}
    X, dY = to_dev(inp["X"], dt), to_dev(inp["dY"], dt)
    Y, dX = empty_dev(X.shape, dt), empty_dev(X.shape, dt)
    L = None
    if inp["lengths"] is not None:
        L = torch.tensor(inp["lengths"], dtype=torch.int32, device="cuda")
    layer.forward(p, X, L, cfg.B, cfg.T, Y, stream_ptr())
    G = None
    if peek_act:
        G = empty_dev((cfg.B, cfg.T, cfg.F), dt)
        assert layer.peek_linear(2, G, stream_ptr()) == G.numel() * G.element_size()
    layer.backward(p, dY, dX, g, stream_ptr())
    torch.cuda.synchronize()
    if own and not keep:
        layer.destroy()
    res = (to_np(Y), to_np(dX), {k: to_np(v) for k, v in g.items()})
    return res + (to_np(G),) if peek_act else res


def avoid_relu_kink(cfg, inp, margin=2e-5, masks=None):
    """relu'(u) jumps at u = 0, so a pre-activation that the fp64 oracle and the fp32 kernel place on
    opposite sides of 0 (they differ by rounding, ~1e-6) would make the two gradients differ by a
    whole term although both are right.  For the fp32 ReLU cases the inputs are therefore moved off
    the kink: bias b1 of every column holding a pre-activation with |u| < margin is shifted by
    4*margin until none is left.  Uses the oracle only.  (The bf16 path cannot avoid this by choosing
    inputs: its pre-activations carry the bf16 rounding of the tensors before them; there the comparison
    is made under the GPU's own decisions, see relu_decisions_of_the_gpu.)"""
    if cfg.act != "relu" or cfg.dtype != "f32":
        return inp
    kw = dict(heads=cfg.H, act=cfg.act, norm=cfg.norm, eps=cfg.eps, causal=cfg.causal, masks=masks)
    for _ in range(50):
        _, c = orc.layer_forward(inp["params"], inp["X"], inp["lengths"], **kw)
        cols = np.unique(np.nonzero(np.abs(c["ffn"]["U"]) < margin)[-1])
        if cols.size == 0:
            return inp
        inp["params"]["b1"][cols] += np.float32(4 * margin)
    raise AssertionError("could not move the pre-activations off the ReLU kink")


def relu_decisions_of_the_gpu(cfg, inp, cache, G_gpu):
    """The bf16 path's ReLU decisions, validated, as a stand-in pre-activation for the oracle's backward.

    relu'(u) = 1[u > 0] is a decision taken in floating point: the bf16 path takes it on its own
    pre-activation, which differs from the fp64 oracle's by the bf16 rounding of the tensors stored before
    it.  Where |u| is below that uncertainty both decisions are valid results of the method, and a single
    flipped decision changes a gradient by a whole term.  So the comparison is made under the GPU's own
    decisions (the sign pattern of the activation output its forward pass recorded), after checking that
    they are valid: a decision may differ from the oracle's only where the oracle's |u| is smaller than
    2^-6 * sqrt(sum_k x_k^2 W_k^2) -- about four standard deviations of what rounding x to bf16 (2^-9
    relative, independent per term) does to the dot product -- and only on a small share of the elements.
    Elements that dropout removed carry no decision (their gradient is zero either way).
    Returns (cache with the decisions put in place of U, share of flipped decisions)."""
    U = cache["ffn"]["U"]
    x, W1 = cache["ffn"]["x"], np.asarray(inp["params"]["W1"], np.float64)
    delta = 2.0 ** -6 * np.sqrt((x * x) @ (W1 * W1).T)
    keep = cache["ffn"].get("keep")
    decided = np.ones(U.shape, bool) if keep is None else np.asarray(keep) > 0
    on_gpu = np.asarray(G_gpu).reshape(U.shape) > 0
    flipped = decided & (on_gpu != (U > 0))
    assert not np.any(flipped & ~(np.abs(U) < delta)), \
        f"{cfg.name}: ReLU decisions differ where the pre-activation is not ambiguous (max |u| {np.abs(U[flipped]).max()})"
    share = float(flipped.sum() / max(1, decided.sum()))
    assert share <= 0.02, f"{cfg.name}: {share:.4f} of the ReLU decisions flipped"
    Umod = np.where(decided, np.where(on_gpu, 1.0, -1.0), U)
    c2 = dict(cache)
    c2["ffn"] = dict(cache["ffn"], U=Umod)
    return c2, share


def check_against_oracle(cfg, inp, tol, dropout=None, test=None):
    masks = None
    if dropout is not None:
        from oracle import dropout as odr
        # the ABI takes the rates as C floats: the oracle gets the same (float32-rounded) values
        dropout = (float(np.float32(dropout[0])), float(np.float32(dropout[1])), dropout[2])
        masks = odr.layer_masks(cfg.B, cfg.T, cfg.D, cfg.H, cfg.F, *dropout)
    inp = avoid_relu_kink(cfg, inp, masks=masks)
    own_decisions = cfg.act == "relu" and cfg.dtype == "bf16"
    res = run_layer_gpu(cfg, inp, dropout=dropout, peek_act=own_decisions)
    Y, dX, g = res[:3]
    kw = dict(heads=cfg.H, act=cfg.act, norm=cfg.norm, eps=cfg.eps, causal=cfg.causal, masks=masks)
    rY, cache = orc.layer_forward(inp["params"], inp["X"], inp["lengths"], **kw)
    extra = {}
    if own_decisions:
        cache, extra["relu_flipped_share"] = relu_decisions_of_the_gpu(cfg, inp, cache, res[3])
    rdX, rg = orc.layer_backward(inp["params"], cache, inp["dY"])
    base = {"Y": rY, "dX": rdX, **{"d" + k: rg[k] for k in PARAM_NAMES}}
    got = {"Y": Y, "dX": dX, **{"d" + k: g[k] for k in PARAM_NAMES}}
    errs = {k: rel_err(got[k], base[k]) for k in base}
    l2 = {k: rel_err_l2(got[k], base[k]) for k in base}
    log_errors(test or cfg.name, errs, l2, extra)
    bad = {k: v for k, v in errs.items() if not v <= tol}
    assert not bad, f"{cfg.name}: above {tol}: {bad}; all: {errs}; {extra}"
    return errs


def _tol(cfg):
    return F32_TOL if cfg.dtype == "f32" else BF16_TOL


@pytest.mark.parametrize("name", ["cfg1_tiny_f32", "cfg2_small_f32", "cfg3_bert_base_bf16"])
@pytest.mark.parametrize("nontrivial", [False, True])
def test_config_full_size(name, nontrivial):
    cfg = CONFIGS[name]
    check_against_oracle(cfg, make_inputs(cfg, seed=0, nontrivial=nontrivial), _tol(cfg))


@pytest.mark.parametrize("seed", [1, 2])
def test_config1_other_seeds(seed):
    cfg = CONFIGS["cfg1_tiny_f32"]
    check_against_oracle(cfg, make_inputs(cfg, seed=seed, nontrivial=True), _tol(cfg))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("norm", ["post", "pre"])
@pytest.mark.parametrize("act", ["relu", "gelu"])
@pytest.mark.parametrize("masked", [False, True])
def test_variants_ragged(dtype, norm, act, masked):
    """Every schedule x activation x mask combination at a shape with ragged tiles (M = 3*37)."""
    cfg = CONFIGS["cfg2_small_f32"].with_(name="ragged", B=3, T=37, D=128, H=2, F=264, dtype=dtype, act=act,
                                          norm=norm, init="xavier")
    inp = make_inputs(cfg, seed=5, nontrivial=True)
    if masked:
        inp["lengths"] = np.array([1, 20, 37], np.int32)
    check_against_oracle(cfg, inp, _tol(cfg))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", [
    dict(B=1, T=1, D=64, H=4, F=64),              # a single token: attention is the identity on V
    dict(B=4, T=1, D=128, H=2, F=256),            # sequences of one token
    dict(B=2, T=9, D=4096, H=16, F=512),          # the largest d_model and head size (256) the layer accepts
    dict(B=1, T=130, D=64, H=1, F=8),             # one head, smallest feed-forward width, two query blocks
    dict(B=5, T=64, D=96, H=6, F=96),             # head size 16: the general attention kernels also in bf16
])
def test_edge_shapes(dtype, shape):
    """Degenerate and extreme shapes, with every sequence but one cut to a single valid key."""
    cfg = CONFIGS["cfg2_small_f32"].with_(name="edge", dtype=dtype, act="gelu", norm="pre",
                                          init="normal0.02" if dtype == "bf16" else "xavier", **shape)
    inp = make_inputs(cfg, seed=8, nontrivial=True)
    lengths = np.ones(cfg.B, np.int32)
    lengths[-1] = cfg.T
    inp["lengths"] = lengths
    check_against_oracle(cfg, inp, _tol(cfg))


def _random_case(k):
    """Case k of a seeded sweep over shapes, types and options (sizes the oracle handles in about a second)."""
    rng = np.random.default_rng(1000 + k)
    dh = int(rng.choice([16, 32, 48, 64, 80, 96, 128]))
    H = int(rng.choice([h for h in (1, 2, 3, 4, 6, 8, 12) if h * dh <= 768]))
    dtype = "bf16" if k % 2 else "f32"
    cfg = CONFIGS["cfg2_small_f32"].with_(
        name=f"random{k}", dtype=dtype, B=int(rng.integers(1, 7)), T=int(rng.integers(1, 301)), D=H * dh, H=H,
        F=8 * int(rng.integers(8, 193)), act=str(rng.choice(["relu", "gelu"])), norm=str(rng.choice(["post", "pre"])),
        init="normal0.02" if dtype == "bf16" else "xavier", causal=bool(rng.integers(0, 2)))
    inp = make_inputs(cfg, seed=2000 + k, nontrivial=True)
    if rng.integers(0, 2):
        inp["lengths"] = rng.integers(1, cfg.T + 1, size=cfg.B).astype(np.int32)
    dropout = (float(rng.choice([0.0, 0.1, 0.3])), float(rng.choice([0.0, 0.1])), 77 + k) if k % 3 == 0 else None
    if dropout is not None and dropout[0] == 0.0 and dropout[1] == 0.0:
        dropout = None
    return cfg, inp, dropout


@pytest.mark.parametrize("k", range(8))
def test_random_midsize_bf16(k):
    """Sizes at which the side stream, the transposed weight copies, the pipelined GEMM variants and the
    split weight-gradient GEMMs are all in play, with ragged token counts."""
    rng = np.random.default_rng(3000 + k)
    D = int(rng.choice([512, 768, 1024]))
    dh = int(rng.choice([64, 128]))
    cfg = CONFIGS["cfg3_bert_base_bf16"].with_(
        name=f"mid{k}", B=int(rng.integers(3, 9)), T=int(rng.integers(150, 400)), D=D, H=D // dh,
        F=64 * int(rng.integers(12, 49)), act=str(rng.choice(["relu", "gelu"])), norm=str(rng.choice(["post", "pre"])),
        causal=bool(rng.integers(0, 2)), len_lo=20, len_hi=150)
    inp = make_inputs(cfg, seed=4000 + k, nontrivial=True)
    dropout = (0.1, 0.1, 5 + k) if k % 4 == 0 else None
    check_against_oracle(cfg, inp, _tol(cfg), dropout=dropout)


@pytest.mark.parametrize("k", range(60))
def test_random_shapes_types_and_options(k):
    """A seeded sweep across head sizes (all multiples of 16 up to 128), ragged token counts, both types,
    both activations and norm placements, causal / padding masks and dropout: whatever kernel the
    selection rules pick for a shape, the layer must match the oracle."""
    cfg, inp, dropout = _random_case(k)
    check_against_oracle(cfg, inp, _tol(cfg), dropout=dropout)


@pytest.mark.parametrize("dtype,norm,act,masked", [("f32", "post", "relu", False), ("f32", "pre", "gelu", True),
                                                   ("bf16", "post", "gelu", True), ("bf16", "pre", "relu", False)])
def test_causal_variants_ragged(dtype, norm, act, masked):
    """The autoregressive variant (key j masked for query i iff j > i) on ragged shapes that span
    several query and key tiles, with and without the key-padding mask on top."""
    cfg = CONFIGS["cfg2_small_f32"].with_(B=3, T=203, D=192, H=3, F=384, dtype=dtype, norm=norm, act=act,
                                          causal=True, len_lo=70 if masked else 0, len_hi=203 if masked else 0,
                                          init="normal0.02" if dtype == "bf16" else "xavier")
    check_against_oracle(cfg, make_inputs(cfg, seed=4, nontrivial=True), _tol(cfg))


def test_causal_config3_full_size():
    """Config 3's shape with the causal mask added: the second workload of the attention kernel."""
    cfg = CONFIGS["cfg3_bert_base_bf16"].with_(causal=True)
    check_against_oracle(cfg, make_inputs(cfg, seed=0, nontrivial=True), _tol(cfg))


def test_causal_rows_do_not_see_the_future():
    """Changing the input from position t0 on must leave every earlier output row bit-identical."""
    cfg = CONFIGS["cfg2_small_f32"].with_(B=2, T=160, dtype="bf16", act="gelu", causal=True, init="normal0.02")
    inp = make_inputs(cfg, seed=5, nontrivial=True)
    Y1 = run_layer_gpu(cfg, inp)[0]
    t0 = 97
    inp2 = dict(inp)
    X2 = inp["X"].copy()
    X2[:, t0:] = np.random.default_rng(1).standard_normal(X2[:, t0:].shape).astype(X2.dtype)
    inp2["X"] = X2
    Y2 = run_layer_gpu(cfg, inp2)[0]
    assert np.array_equal(Y1[:, :t0], Y2[:, :t0])
    assert not np.array_equal(Y1[:, t0:], Y2[:, t0:])


@pytest.mark.parametrize("dtype,norm,act,masked,causal", [("f32", "post", "relu", False, False),
                                                          ("f32", "pre", "gelu", True, True),
                                                          ("bf16", "post", "gelu", True, False),
                                                          ("bf16", "pre", "relu", False, True)])
def test_dropout_variants_ragged(dtype, norm, act, masked, causal):
    """All four dropout sites on, ragged shapes spanning several tiles; the oracle regenerates the same
    masks from the seed, so outputs and every gradient must agree to the usual tolerance."""
    cfg = CONFIGS["cfg2_small_f32"].with_(B=3, T=203, D=192, H=3, F=392, dtype=dtype, norm=norm, act=act,
                                          causal=causal, len_lo=70 if masked else 0, len_hi=203 if masked else 0,
                                          init="normal0.02" if dtype == "bf16" else "xavier")
    check_against_oracle(cfg, make_inputs(cfg, seed=6, nontrivial=True), _tol(cfg), dropout=(0.15, 0.3, 0xABCDEF0123456789))


def test_dropout_config3_full_size():
    """Config 3's shape in training mode (rate 0.1 at every site)."""
    cfg = CONFIGS["cfg3_bert_base_bf16"]
    check_against_oracle(cfg, make_inputs(cfg, seed=0, nontrivial=True), _tol(cfg), dropout=(0.1, 0.1, 2026))


def test_dropout_settings_belong_to_the_recorded_forward():
    """Changing the settings between a forward and its backward must not affect that backward; rate 0
    is bit-identical to a layer that never heard of dropout; a new seed changes the result."""
    from paper_2201_12465_amd import binding as b
    cfg = CONFIGS["cfg2_small_f32"].with_(dtype="bf16", act="gelu", init="normal0.02")
    inp = make_inputs(cfg, seed=2, nontrivial=True)
    ref = run_layer_gpu(cfg, inp, dropout=(0.2, 0.2, 11))
    torch = torch_mod()
    layer = b.Layer(cfg.B, cfg.T, cfg.D, cfg.H, cfg.F, cfg.act, cfg.norm, cfg.dtype, cfg.eps)
    p = {k: to_dev(v, cfg.dtype) for k, v in inp["params"].items()}
    g = {k: empty_dev(v.shape, cfg.dtype) for k, v in inp["params"].items()}
    X, dY = to_dev(inp["X"], cfg.dtype), to_dev(inp["dY"], cfg.dtype)
    Y, dX = empty_dev(X.shape, cfg.dtype), empty_dev(X.shape, cfg.dtype)
    layer.set_dropout(0.2, 0.2, 11)
    layer.forward(p, X, None, cfg.B, cfg.T, Y, stream_ptr())
    layer.set_dropout(0.5, 0.0, 99)                     # must only affect the NEXT forward
    layer.backward(p, dY, dX, g, stream_ptr())
    torch.cuda.synchronize()
    assert np.array_equal(to_np(Y), ref[0]) and np.array_equal(to_np(dX), ref[1])
    for k in PARAM_NAMES:
        assert np.array_equal(to_np(g[k]), ref[2][k]), k
    layer.destroy()
    off = run_layer_gpu(cfg, inp, dropout=(0.0, 0.0, 5))
    plain = run_layer_gpu(cfg, inp)
    assert np.array_equal(off[0], plain[0]) and np.array_equal(off[1], plain[1])
    other = run_layer_gpu(cfg, inp, dropout=(0.2, 0.2, 12))
    assert not np.array_equal(other[0], ref[0])
    with pytest.raises(b.FlError) as e:
        b.Layer(cfg.B, cfg.T, cfg.D, cfg.H, cfg.F).set_dropout(1.0, 0.0, 0)
    assert e.value.status == b.FL_ERR_INVALID_ARG


def test_config4_full_size():
    """Config 4 as the benchmark spec states it (B=8, T=1000, 4 heads of 192, ReLU, masked)."""
    cfg = CONFIGS["cfg4_speech_bf16"]
    check_against_oracle(cfg, make_inputs(cfg, seed=0), _tol(cfg))


def test_speech_shape_reduced():
    """Config 4's head size (192) and a long, masked, non-tile-multiple sequence, at reduced batch."""
    cfg = CONFIGS["cfg4_speech_bf16"].with_(B=2, T=333, len_lo=150, len_hi=333)
    check_against_oracle(cfg, make_inputs(cfg, seed=0, nontrivial=True), _tol(cfg))


def test_vit_stack_reduced():
    """Config 5's chain (pre-LN, GELU, T=197) through the same layer calls: 3 layers, batch 4."""
    _run_stack(CONFIGS["cfg5_vit_b16_bf16"].with_(B=4, layers=3), nontrivial=True, test="cfg5_reduced_3_layers")


def test_config5_full_stack():
    """Config 5 as the benchmark spec states it: 12 pre-LN layers, B=64, T=197.  Two comparisons, both at the
    flat bf16 tolerance: (1) the chain end to end -- final Y, dX at the stack input and all 12 layers'
    parameter gradients against the oracle's chain; (2) every layer on its own -- the oracle is given the
    very input and upstream gradient the GPU's layer l received (the GPU's own bf16 tensors), so that each
    layer's Y, dX and 12 gradients are checked without the error the chain has built up before it.
    Run once with every backward joining the side stream itself and once the way the benchmark runs the
    stack (one join per layer after the last backward)."""
    _run_stack(CONFIGS["cfg5_vit_b16_bf16"], nontrivial=False, deferred_too=True, test="cfg5_vit_b16_bf16")


# The chain of 12 layer calls hands bf16 tensors from call to call: against the un-rounded fp64 chain the
# residual stream and the gradient stream are each rounded 24 times, whatever the kernels do, and those
# roundings add up like a random walk (per layer: 0.005; chain: 0.017 on Y, 0.018 on dX).  The chain is held
# to the same flat tolerance as a single layer; so is every tensor of every single layer.


def _run_stack(cfg, nontrivial, deferred_too=False, test=None):
    from paper_2201_12465_amd import binding as b
    torch = torch_mod()
    inp = make_stack_inputs(cfg, seed=0, nontrivial=nontrivial)
    dt = cfg.dtype
    kw = dict(heads=cfg.H, act=cfg.act, norm=cfg.norm, eps=cfg.eps)
    rY, rdX, rg = orc.stack_forward_backward(inp["params"], inp["X"], inp["dY"], None, **kw)
    P = [{k: to_dev(v, dt) for k, v in p.items()} for p in inp["params"]]
    for deferred in ([False, True] if deferred_too else [False]):
        layers = [b.Layer(cfg.B, cfg.T, cfg.D, cfg.H, cfg.F, cfg.act, cfg.norm, dt, cfg.eps) for _ in range(cfg.layers)]
        G = [{k: empty_dev(v.shape, dt) for k, v in p.items()} for p in inp["params"]]
        acts = [to_dev(inp["X"], dt)] + [empty_dev(inp["X"].shape, dt) for _ in range(cfg.layers)]
        grads = [empty_dev(inp["X"].shape, dt) for _ in range(cfg.layers)] + [to_dev(inp["dY"], dt)]
        s = stream_ptr()
        for ly in layers:
            ly.set_deferred_join(deferred)
        for l in range(cfg.layers):
            layers[l].forward(P[l], acts[l], None, cfg.B, cfg.T, acts[l + 1], s)
        for l in reversed(range(cfg.layers)):
            layers[l].backward(P[l], grads[l + 1], grads[l], G[l], s)
        for ly in layers:
            ly.join(s)   # nothing to do unless deferred
        torch.cuda.synchronize()
        for L in layers:
            L.destroy()
        # (1) the chain end to end
        pairs = {"Y": (to_np(acts[-1]), rY), "dX": (to_np(grads[0]), rdX)}
        for l in range(cfg.layers):
            for k in PARAM_NAMES:
                pairs[f"L{l}.d{k}"] = (to_np(G[l][k]), rg[l][k])
        errs = {k: rel_err(a, r) for k, (a, r) in pairs.items()}
        l2 = {k: rel_err_l2(a, r) for k, (a, r) in pairs.items()}
        log_errors(f"{test}/chain/deferred={deferred}", errs, l2)
        print(f"stack of {cfg.layers} (deferred join: {deferred}): chain, largest error {max(errs.values()):.4f}")
        bad = {k: v for k, v in errs.items() if not v <= BF16_TOL}
        assert not bad, ("chain", deferred, BF16_TOL, bad)
        if deferred:
            continue   # same kernels, same bits (test_deferred_join_changes_no_bit): the per-layer pass is not repeated
        # (2) every layer on its own, fed what the GPU's layer was fed
        worst = {}
        for l in range(cfg.layers):
            x_l, dy_l = to_np(acts[l]), to_np(grads[l + 1])
            oY, odX, og = orc.layer_forward_backward(inp["params"][l], x_l, dy_l, None, **kw)
            pl = {"Y": (to_np(acts[l + 1]), oY), "dX": (to_np(grads[l]), odX)}
            pl.update({"d" + k: (to_np(G[l][k]), og[k]) for k in PARAM_NAMES})
            e_l = {k: rel_err(a, r) for k, (a, r) in pl.items()}
            l2_l = {k: rel_err_l2(a, r) for k, (a, r) in pl.items()}
            log_errors(f"{test}/layer{l}", e_l, l2_l)
            bad = {k: v for k, v in e_l.items() if not v <= BF16_TOL}
            assert not bad, ("layer", l, BF16_TOL, bad)
            worst[l] = max(e_l.values())
        print(f"stack of {cfg.layers}: per-layer largest errors {worst}")


@pytest.mark.parametrize("join", ["explicit", "next-forward", "other-stream"])
def test_deferred_join_changes_no_bit(join):
    """A stack whose layers leave the side-stream join to fl_layer_join (or to their next forward) produces
    the same bits as one that joins in every backward; two steps, so that buffers are reused across them."""
    from paper_2201_12465_amd import binding as b
    torch = torch_mod()
    cfg = CONFIGS["cfg5_vit_b16_bf16"].with_(B=8, layers=3)
    inp = make_stack_inputs(cfg, seed=1, nontrivial=True)
    dt = cfg.dtype

    def run(deferred):
        layers = [b.Layer(cfg.B, cfg.T, cfg.D, cfg.H, cfg.F, cfg.act, cfg.norm, dt, cfg.eps) for _ in range(cfg.layers)]
        for ly in layers:
            ly.set_deferred_join(deferred)
        P = [{k: to_dev(v, dt) for k, v in p.items()} for p in inp["params"]]
        G = [{k: empty_dev(v.shape, dt) for k, v in p.items()} for p in inp["params"]]
        acts = [to_dev(inp["X"], dt)] + [empty_dev(inp["X"].shape, dt) for _ in range(cfg.layers)]
        grads = [empty_dev(inp["X"].shape, dt) for _ in range(cfg.layers)] + [to_dev(inp["dY"], dt)]
        s = stream_ptr()
        other = torch.cuda.Stream()
        for step in range(2):
            for l in range(cfg.layers):
                layers[l].forward(P[l], acts[l], None, cfg.B, cfg.T, acts[l + 1], s)   # joins what step 0 left open
            for l in reversed(range(cfg.layers)):
                layers[l].backward(P[l], grads[l + 1], grads[l], G[l], s)
            if deferred and join == "explicit":
                for ly in layers:
                    ly.join(s)
            if deferred and join == "other-stream" and step == 1:
                for ly in layers:
                    ly.join(other.cuda_stream)
                other.synchronize()
        if deferred and join == "next-forward":
            for ly in layers:   # destroy joins too; here the results are read first
                ly.join(s)
        torch.cuda.synchronize()
        out = [to_np(acts[-1]), to_np(grads[0])] + [to_np(G[l][k]) for l in range(cfg.layers) for k in PARAM_NAMES]
        for ly in layers:
            ly.destroy()
        return out

    ref, got = run(False), run(True)
    for i, (r, g) in enumerate(zip(ref, got)):
        assert np.array_equal(r, g), (join, i)


def test_deferred_join_lets_the_caller_reuse_the_upstream_gradient_buffer():
    """A stack that ping-pongs TWO gradient buffers: layer l writes its dX into the buffer that held the dY of
    layer l+1.  With the join deferred, layer l+1's weight-gradient kernels (which read that dY on the side
    stream) must be done before layer l's chain overwrites it.  Same bits as the run that joins in every
    backward and keeps one buffer per layer."""
    from paper_2201_12465_amd import binding as b
    torch = torch_mod()
    cfg = CONFIGS["cfg5_vit_b16_bf16"].with_(B=16, layers=4)
    inp = make_stack_inputs(cfg, seed=2, nontrivial=True)
    dt = cfg.dtype

    def run(deferred):
        layers = [b.Layer(cfg.B, cfg.T, cfg.D, cfg.H, cfg.F, cfg.act, cfg.norm, dt, cfg.eps) for _ in range(cfg.layers)]
        for ly in layers:
            ly.set_deferred_join(deferred)
        P = [{k: to_dev(v, dt) for k, v in p.items()} for p in inp["params"]]
        G = [{k: empty_dev(v.shape, dt) for k, v in p.items()} for p in inp["params"]]
        acts = [to_dev(inp["X"], dt)] + [empty_dev(inp["X"].shape, dt) for _ in range(cfg.layers)]
        if deferred:
            ping = [to_dev(inp["dY"], dt), empty_dev(inp["X"].shape, dt)]
            grads = [ping[(cfg.layers - l) % 2] for l in range(cfg.layers + 1)]   # grads[layers] = dY
        else:
            grads = [empty_dev(inp["X"].shape, dt) for _ in range(cfg.layers)] + [to_dev(inp["dY"], dt)]
        s = stream_ptr()
        for step in range(2):
            if deferred and step:
                grads[cfg.layers].copy_(to_dev(inp["dY"], dt))   # the first step's chain has overwritten it
            for l in range(cfg.layers):
                layers[l].forward(P[l], acts[l], None, cfg.B, cfg.T, acts[l + 1], s)
            for l in reversed(range(cfg.layers)):
                layers[l].backward(P[l], grads[l + 1], grads[l], G[l], s)
            for ly in layers:
                ly.join(s)
        torch.cuda.synchronize()
        out = [to_np(grads[0])] + [to_np(G[l][k]) for l in range(cfg.layers) for k in PARAM_NAMES]
        for ly in layers:
            ly.destroy()
        return out

    ref, got = run(False), run(True)
    for i, (r, g) in enumerate(zip(ref, got)):
        assert np.array_equal(r, g), i


def test_lengths_outside_the_valid_range():
    """1 <= lengths[b] <= T is a precondition.  The kernels treat a length outside it as the nearest valid one
    (no read past a sequence, no 0/0 row); with FL_DEBUG=1 in the environment forward checks the lengths on
    the host and refuses them, and hands out NaN-filled buffers without changing any result."""
    import os
    from paper_2201_12465_amd import binding as b
    torch = torch_mod()
    for dtype in ("f32", "bf16"):
        cfg = CONFIGS["cfg2_small_f32"].with_(B=3, T=70, D=128, H=2, F=256, dtype=dtype, act="gelu",
                                              init="normal0.02" if dtype == "bf16" else "xavier")
        inp = make_inputs(cfg, seed=9, nontrivial=True)
        inp["lengths"] = np.array([0, 75, 33], np.int32)
        clamped = dict(inp, lengths=np.array([1, 70, 33], np.int32))
        got, want = run_layer_gpu(cfg, inp), run_layer_gpu(cfg, clamped)
        assert np.array_equal(got[0], want[0]) and np.array_equal(got[1], want[1])
        for k in PARAM_NAMES:
            assert np.array_equal(got[2][k], want[2][k]), k
        os.environ["FL_DEBUG"] = "1"
        try:
            with pytest.raises(b.FlError) as e:
                run_layer_gpu(cfg, inp)
            assert e.value.status == b.FL_ERR_INVALID_ARG and "lengths[0] = 0" in str(e.value)
            poisoned = run_layer_gpu(cfg, clamped)
        finally:
            del os.environ["FL_DEBUG"]
        assert np.array_equal(poisoned[0], want[0]) and np.array_equal(poisoned[1], want[1])
        for k in PARAM_NAMES:
            assert np.array_equal(poisoned[2][k], want[2][k]), k
    torch.cuda.synchronize()
    assert b.alloc_stats()["live_bytes"] == 0


def test_masked_keys_get_exactly_zero_influence():
    """Changing X at a padded position changes only that position's output row."""
    cfg = CONFIGS["cfg2_small_f32"].with_(B=2, T=40, D=64, H=4, F=128)
    inp = make_inputs(cfg, seed=3, nontrivial=True)
    inp["lengths"] = np.array([17, 40], np.int32)
    Y0, _, _ = run_layer_gpu(cfg, inp)
    inp2 = dict(inp)
    X2 = inp["X"].copy()
    X2[0, 30] += 3.0
    inp2["X"] = X2
    Y1, _, _ = run_layer_gpu(cfg, inp2)
    rows = [i for i in range(cfg.T) if i != 30]
    assert np.array_equal(Y0[0, rows], Y1[0, rows])
    assert np.array_equal(Y0[1], Y1[1])
    assert not np.array_equal(Y0[0, 30], Y1[0, 30])


def test_steady_state_has_no_device_mallocs_and_is_deterministic():
    from paper_2201_12465_amd import binding as b
    cfg = CONFIGS["cfg2_small_f32"]
    inp = make_inputs(cfg, seed=0)
    layer = b.Layer(cfg.B, cfg.T, cfg.D, cfg.H, cfg.F, cfg.act, cfg.norm, cfg.dtype, cfg.eps)
    outs = []
    for it in range(4):
        outs.append(run_layer_gpu(cfg, inp, layer=layer))
        if it == 1:
            warm = b.alloc_stats()
    layer.destroy()     # the handle keeps a few hundred bytes of split-k counters while it lives
    end = b.alloc_stats()
    assert end["backing_mallocs"] == warm["backing_mallocs"], (warm, end)
    assert end["live_bytes"] == 0
    assert end["cache_hits"] > warm["cache_hits"]
    for o in outs[1:]:
        assert np.array_equal(o[0], outs[0][0]) and np.array_equal(o[1], outs[0][1])
        for k in PARAM_NAMES:
            assert np.array_equal(o[2][k], outs[0][2][k]), k


def _classes_of_one_step(cfg, inp, layer=None):
    from paper_2201_12465_amd import binding as b
    b.prof_enable("all")
    try:
        res = run_layer_gpu(cfg, inp, layer=layer)
        prof = b.prof_collect()
    finally:
        b.prof_enable(None)
    return res, {k: v["launches"] for k, v in prof.items()}


@pytest.mark.parametrize("norm", ["post", "pre"])
@pytest.mark.parametrize("overlap", [True, False])
def test_input_gradients_take_transposed_weight_copies_where_it_pays(overlap, norm):
    """bf16 layers of middling size leave W^T behind in forward and run dx = dy (W^T)^T on the kernel for
    operands that are contiguous along the contraction; results stay within the oracle's tolerance
    (ragged token count, so edge tiles are exercised), small and fp32 layers keep dx = dy W."""
    from paper_2201_12465_amd import binding as b
    cfg = CONFIGS["cfg3_bert_base_bf16"].with_(B=5, T=120, D=512, H=8, F=1088, len_lo=30, len_hi=120, norm=norm)
    inp = make_inputs(cfg, seed=11, nontrivial=True)
    b.set_grad_overlap(overlap)
    try:
        _, launches = _classes_of_one_step(cfg, inp)
        check_against_oracle(cfg, inp, _tol(cfg))
    finally:
        b.set_grad_overlap(True)
    assert launches.get("wt_transpose") == 1 and "gemm_nn" not in launches and launches["gemm_nt"] == 8
    small = CONFIGS["cfg3_bert_base_bf16"].with_(B=2, T=64, D=256, H=4, F=512, len_lo=10, len_hi=64)
    _, launches = _classes_of_one_step(small, make_inputs(small, seed=2))
    assert "wt_transpose" not in launches and launches["gemm_nn"] == 4
    _, launches = _classes_of_one_step(CONFIGS["cfg2_small_f32"], make_inputs(CONFIGS["cfg2_small_f32"], seed=2))
    assert "wt_transpose" not in launches and launches["gemm_nn"] == 4
    assert b.alloc_stats()["live_bytes"] == 0


def test_forward_without_backward_releases_the_transposed_copies():
    """Two forwards in a row on one handle (the first recording is dropped while its copies may still be
    in flight on the side stream), then a backward: same result as a fresh handle, nothing left allocated."""
    from paper_2201_12465_amd import binding as b
    cfg = CONFIGS["cfg3_bert_base_bf16"].with_(B=8)
    inp = make_inputs(cfg, seed=4, nontrivial=True)
    ref = run_layer_gpu(cfg, inp)
    torch = torch_mod()
    dt = cfg.dtype
    layer = b.Layer(cfg.B, cfg.T, cfg.D, cfg.H, cfg.F, cfg.act, cfg.norm, dt, cfg.eps)
    p = {k: to_dev(v, dt) for k, v in inp["params"].items()}
    X = to_dev(inp["X"], dt)
    Y = empty_dev(X.shape, dt)
    L = torch.tensor(inp["lengths"], dtype=torch.int32, device="cuda")
    layer.forward(p, X, L, cfg.B, cfg.T, Y, stream_ptr())
    res = run_layer_gpu(cfg, inp, layer=layer)
    layer.forward(p, X, L, cfg.B, cfg.T, Y, stream_ptr())   # recorded, never replayed: destroy must clean up
    layer.destroy()
    torch.cuda.synchronize()
    assert np.array_equal(res[0], ref[0]) and np.array_equal(res[1], ref[1])
    for k in PARAM_NAMES:
        assert np.array_equal(res[2][k], ref[2][k]), k
    assert b.alloc_stats()["live_bytes"] == 0


@pytest.mark.parametrize("name", ["cfg1_tiny_f32", "cfg3_bert_base_bf16"])
def test_step_can_be_captured_in_a_graph_and_replayed(name):
    """A caller may capture forward + backward in a HIP graph once the allocator's cache is warm (no
    device allocation happens during capture; the side streams join the capture through the fork
    events).  Every replay, with eager work and synchronisation in between, must reproduce the eager
    result bit for bit."""
    from paper_2201_12465_amd import binding as b
    torch = torch_mod()
    cfg = CONFIGS[name].with_(B=min(CONFIGS[name].B, 8))
    inp = make_inputs(cfg, seed=6, nontrivial=True)
    dt = cfg.dtype
    layer = b.Layer(cfg.B, cfg.T, cfg.D, cfg.H, cfg.F, cfg.act, cfg.norm, dt, cfg.eps)
    p = {k: to_dev(v, dt) for k, v in inp["params"].items()}
    g = {k: empty_dev(v.shape, dt) for k, v in inp["params"].items()}
    X, dY = to_dev(inp["X"], dt), to_dev(inp["dY"], dt)
    Y, dX = empty_dev(X.shape, dt), empty_dev(X.shape, dt)
    L = torch.tensor(inp["lengths"], dtype=torch.int32, device="cuda") if inp["lengths"] is not None else None
    s = torch.cuda.Stream()

    def step():
        layer.forward(p, X, L, cfg.B, cfg.T, Y, s.cuda_stream)
        layer.backward(p, dY, dX, g, s.cuda_stream)

    def snapshot():
        torch.cuda.synchronize()
        return [Y.clone(), dX.clone()] + [g[k].clone() for k in PARAM_NAMES]

    with torch.cuda.stream(s):
        for _ in range(3):          # warms the cache of this stream and of the side streams
            step()
        ref = snapshot()
        mallocs = b.alloc_stats()["backing_mallocs"]
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=s):
            step()
        assert b.alloc_stats()["backing_mallocs"] == mallocs
        for rep in range(3):
            for t in [Y, dX] + list(g.values()):
                t.fill_(float("nan"))
            torch.cuda.synchronize()
            graph.replay()
            got = snapshot()
            assert all(torch.equal(a, r) for a, r in zip(got, ref)), rep
            (X.float() @ X.float().transpose(1, 2)).sum().item()     # unrelated eager work between replays
        step()                       # and the handle still works eagerly afterwards
        got = snapshot()
        assert all(torch.equal(a, r) for a, r in zip(got, ref))
    del graph
    layer.destroy()
    assert b.alloc_stats()["live_bytes"] == 0


@pytest.mark.parametrize("name", ["cfg2_small_f32", "cfg3_bert_base_bf16"])
def test_side_stream_for_parameter_gradients_changes_no_bit(name):
    """The parameter-gradient kernels run beside the input-gradient chain on a side stream; with that
    switched off everything runs in order on the caller's stream.  Same kernels, same summation order:
    the two must agree bit for bit, also when gradients are accumulated over two backward passes."""
    from paper_2201_12465_amd import binding as b
    cfg = CONFIGS[name]
    inp = make_inputs(cfg, seed=3)
    ref = None
    try:
        for overlap in (True, False, True):
            b.set_grad_overlap(overlap)
            layer = b.Layer(cfg.B, cfg.T, cfg.D, cfg.H, cfg.F, cfg.act, cfg.norm, cfg.dtype, cfg.eps)
            for _ in range(2):                      # the second pass reuses cached blocks of both streams
                res = run_layer_gpu(cfg, inp, layer=layer)
            layer.destroy()
            ref = ref or res
            assert np.array_equal(res[0], ref[0]) and np.array_equal(res[1], ref[1]), overlap
            for k in PARAM_NAMES:
                assert np.array_equal(res[2][k], ref[2][k]), (overlap, k)
    finally:
        b.set_grad_overlap(True)
    assert b.alloc_stats()["live_bytes"] == 0


def test_side_stream_repeated_steps_stay_bit_identical():
    """Thirty back-to-back training steps on one handle with the side stream on (events and cached
    blocks of both streams are reused every step, nothing synchronises the host in between): every
    step's gradients must equal the first step's."""
    from paper_2201_12465_amd import binding as b
    torch = torch_mod()
    cfg = CONFIGS["cfg3_bert_base_bf16"].with_(B=8)
    inp = make_inputs(cfg, seed=1, nontrivial=True)
    dt = cfg.dtype
    layer = b.Layer(cfg.B, cfg.T, cfg.D, cfg.H, cfg.F, cfg.act, cfg.norm, dt, cfg.eps)
    p = {k: to_dev(v, dt) for k, v in inp["params"].items()}
    X, dY = to_dev(inp["X"], dt), to_dev(inp["dY"], dt)
    L = torch.tensor(inp["lengths"], dtype=torch.int32, device="cuda")
    outs = []
    for it in range(30):
        g = {k: empty_dev(v.shape, dt) for k, v in inp["params"].items()}
        Y, dX = empty_dev(X.shape, dt), empty_dev(X.shape, dt)
        layer.forward(p, X, L, cfg.B, cfg.T, Y, stream_ptr())
        layer.backward(p, dY, dX, g, stream_ptr())
        outs.append((Y, dX, g))                      # kept alive: no reuse of these buffers by torch
    torch.cuda.synchronize()
    layer.destroy()
    ref = outs[0]
    for it, (Y, dX, g) in enumerate(outs[1:], 1):
        assert torch.equal(Y, ref[0]) and torch.equal(dX, ref[1]), it
        for k in PARAM_NAMES:
            assert torch.equal(g[k], ref[2][k]), (it, k)


def test_allocation_trace_names_the_operator_of_every_buffer():
    """Section 5.2.2 telemetry: each intermediate buffer of one forward + backward is tied to the
    operator that asked for it, and everything handed out comes back."""
    from paper_2201_12465_amd import binding as b
    cfg = CONFIGS["cfg2_small_f32"]
    inp = make_inputs(cfg, seed=0)
    layer = b.Layer(cfg.B, cfg.T, cfg.D, cfg.H, cfg.F, cfg.act, cfg.norm, cfg.dtype, cfg.eps)
    run_layer_gpu(cfg, inp, layer=layer)                  # warm the cache
    b.alloc_trace_enable(1024)
    try:
        run_layer_gpu(cfg, inp, layer=layer)
        ev = b.alloc_trace_read(1024)
    finally:
        b.alloc_trace_enable(0)
        layer.destroy()
    allocs = [e for e in ev if e["kind"] != "release"]
    assert allocs and all(e["kind"] == "from_cache" for e in allocs)       # steady state: no device allocation
    assert all(e["op"] != "none" for e in allocs)
    fwd = [e for e in allocs if e["op"].endswith("_fwd")]
    M, el = cfg.B * cfg.T, 4
    # forward, post-LN with ReLU: qkv, attention output, out-projection, LN1, the two feed-forward linears
    # (LN2 writes the caller's Y); the log-sum-exp and LayerNorm statistics are the smaller buffers
    assert [(e["op"], e["node"]) for e in fwd if e["requested"] >= M * cfg.D * el] == [
        ("linear_fwd", 0), ("attention_fwd", 1), ("linear_fwd", 2), ("layernorm_fwd", 3),
        ("linear_fwd", 4), ("linear_fwd", 5)]
    assert fwd[0]["requested"] == M * 3 * cfg.D * el
    assert [e["requested"] for e in fwd if e["node"] == 4] == [M * cfg.F * el]
    assert sorted(e["requested"] for e in fwd if e["requested"] < M * cfg.D * el) == sorted(
        [cfg.B * cfg.H * cfg.T * 4, 2 * M * 4, 2 * M * 4])
    assert {e["op"] for e in allocs} >= {"linear_bwd", "attention_bwd", "layernorm_bwd"}
    # every block handed out during the traced pass is given back during it, under the tag it was handed out with
    open_ = {}
    for e in ev:
        if e["kind"] == "release":
            if e["ptr"] in open_:
                a = open_.pop(e["ptr"])
                assert (a["op"], a["node"]) == (e["op"], e["node"]) and a["granted"] == e["granted"]
        else:
            assert e["ptr"] not in open_ and e["granted"] >= e["requested"]
            open_[e["ptr"]] = e
    assert open_ == {}


def test_error_paths():
    from paper_2201_12465_amd import binding as b
    cfg = CONFIGS["cfg1_tiny_f32"]
    inp = make_inputs(cfg, seed=0)
    layer = b.Layer(cfg.B, cfg.T, cfg.D, cfg.H, cfg.F)
    p = {k: to_dev(v, "f32") for k, v in inp["params"].items()}
    g = {k: empty_dev(v.shape, "f32") for k, v in inp["params"].items()}
    X = to_dev(inp["X"], "f32")
    Y = empty_dev(X.shape, "f32")
    with pytest.raises(b.FlError) as e:
        layer.backward(p, X, Y, g, stream_ptr())          # nothing recorded yet
    assert e.value.status == b.FL_ERR_STATE
    with pytest.raises(b.FlError) as e:
        layer.forward(p, X, None, cfg.B + 1, cfg.T, Y, stream_ptr())
    assert e.value.status == b.FL_ERR_INVALID_ARG
    with pytest.raises(b.FlError) as e:
        layer.forward(p, X.data_ptr() + 4, None, cfg.B, cfg.T, Y, stream_ptr())
    assert e.value.status == b.FL_ERR_UNSUPPORTED
    layer.forward(p, X, None, cfg.B, cfg.T, Y, stream_ptr())
    layer.backward(p, X, Y, g, stream_ptr())
    with pytest.raises(b.FlError) as e:
        layer.backward(p, X, Y, g, stream_ptr())          # the tape was consumed
    assert e.value.status == b.FL_ERR_STATE
    torch_mod().cuda.synchronize()
    layer.destroy()
    assert b.alloc_stats()["live_bytes"] == 0
